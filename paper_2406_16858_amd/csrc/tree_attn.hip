// Tree attention of the verification pass (Section 4.2 of the EAGLE-2 paper: every tree
// row sees the whole KV prefix plus exactly its ancestors and itself among the tree keys).
//
// bf16 path: split-KV attention on the matrix cores.  The prefix keys of a sequence are cut
// into chunks of `chunk` keys; a workgroup handles one chunk for one KV head and one block of
// query rows, and the workgroups of a sequence's last chunk go on to its N tree keys.  All
// Hq/Hkv * N query rows of a KV head share each K/V tile.  Both products are computed
// transposed so that every lane keeps a single query row:
//     S^T = K . Q^T   (A = K tile from LDS, B = Q fragments held in registers)
//     O^T = V^T . P^T (A = V tile from LDS through the transposing read, B = the probabilities just computed)
// The output registers of the first product are, lane for lane, the B operand of the
// second (the contraction index of an MFMA may be permuted freely as long as A and B
// agree), so P never goes through LDS.  The ancestor bitmask is applied to the tree
// keys only.  The exp2 arguments are taken against a per-row reference that follows the running
// maximum lazily (see the softmax step in compute); a second kernel combines the chunks'
// (reference, sum, O) triples.
// The prefix keys/values may also be 8-bit E4M3 codes with per-head scales (KV8 instantiations).
//
// fp32 path: a plain one-query-row-per-workgroup kernel in float32 (small shapes only).

#include "common.h"

namespace eagle2 {

constexpr int TA_THREADS = 256;
constexpr int TA_KEYS = 64;              // keys per tile
constexpr float NEG_BIG = -1.0e30f;

struct SeqChunk { int b; int c; int nc; long long off; long long P; int first; };

// Keys of sequence b's prefix: its whole region of the KV buffer, or the filled part of it when
// the caller keeps a pre-allocated cache (kv_len, clamped to the region).
__device__ __forceinline__ long long prefix_keys(int b, const long long* kv_offsets, const int* kv_len) {
    const long long region = kv_offsets[b + 1] - kv_offsets[b];
    if (kv_len == nullptr) return region;
    const long long n = kv_len[b];
    return n < 0 ? 0 : (n < region ? n : region);
}
// Maps a flat chunk index to (sequence, chunk); sequence b has max(1, ceil(P_b / chunk)) chunks of
// prefix keys, and the last of them also takes the sequence's tree keys.
__device__ __forceinline__ int seq_chunks(long long P, int chunk) {
    const int n = (int)((P + chunk - 1) / chunk);
    return n < 1 ? 1 : n;
}
// The chunk counts of up to 64 sequences at a time are taken by the lanes of a wave (one vector load each
// instead of a chain of dependent scalar loads per sequence) and summed with a shuffle scan; the results
// are the same in every lane.  Every lane of the wave must be active.
__device__ __forceinline__ int wave_inclusive_sum(int v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(v, o, 64);
        if (lane >= o) v += u;
    }
    return v;
}
__device__ __forceinline__ long long read_lane_ll(long long v, int l) {
    const unsigned lo = (unsigned)read_lane_dyn((int)(unsigned)v, l), hi = (unsigned)read_lane_dyn((int)(unsigned)((unsigned long long)v >> 32), l);
    return (long long)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ bool locate_chunk(int flat, int B, int chunk, const long long* kv_offsets, const int* kv_len, SeqChunk& sc) {
    if (B == 1) {                                      // one sequence: nothing to search
        const long long P = prefix_keys(0, kv_offsets, kv_len);
        const int nc = seq_chunks(P, chunk);
        if (flat >= nc) return false;
        sc.b = 0; sc.c = flat; sc.nc = nc; sc.off = kv_offsets[0]; sc.P = P; sc.first = 0;
        return true;
    }
    const int lane = threadIdx.x & 63;
    int before = 0;                                    // chunks of the sequences in earlier batches of 64
    for (int b0 = 0; b0 < B; b0 += 64) {
        const int b = b0 + lane;
        long long off = 0, P = 0;
        int nc = 0;
        if (b < B) { off = kv_offsets[b]; P = prefix_keys(b, kv_offsets, kv_len); nc = seq_chunks(P, chunk); }
        const int incl = wave_inclusive_sum(nc, lane);
        const unsigned long long holds = __ballot(before + incl > flat);   // lanes whose sequence ends beyond the chunk
        if (holds) {
            const int l = __ffsll((long long)holds) - 1;
            sc.b = b0 + l;
            sc.nc = read_lane_dyn(nc, l);
            sc.first = before + read_lane_dyn(incl, l) - sc.nc;
            sc.c = flat - sc.first;
            sc.off = read_lane_ll(off, l);
            sc.P = read_lane_ll(P, l);
            return true;
        }
        before += read_lane_dyn(incl, 63);
    }
    return false;
}
__device__ __forceinline__ void locate_seq(int b, int chunk, const long long* kv_offsets, const int* kv_len, int& first, int& nc) {
    first = 0;
    if (b == 0) { nc = seq_chunks(prefix_keys(0, kv_offsets, kv_len), chunk); return; }
    const int lane = threadIdx.x & 63;
    nc = 0;
    for (int b0 = 0; b0 <= b; b0 += 64) {
        const int i = b0 + lane;
        const int n = i <= b ? seq_chunks(prefix_keys(i, kv_offsets, kv_len), chunk) : 0;
        const int incl = wave_inclusive_sum(n, lane);
        if (b - b0 < 64) {
            nc = read_lane_dyn(n, b - b0);
            first += read_lane_dyn(incl, b - b0) - nc;
        } else {
            first += read_lane_dyn(incl, 63);
        }
    }
}

template <int DH> __device__ __forceinline__ int k_swz(int row) { return DH == 128 ? (row & 15) : ((row >> 1) & 7); }
// V rows are cut into 32-byte granules (16 dh: what one PV fragment covers); a row's granules are
// permuted by its key index so that the four key rows one transpose read touches fall in different banks
template <int DH> __device__ __forceinline__ int v_swz(int key) { return key & (DH / 16 - 1); }
// Tells the compiler that a pointer is the same in every lane, so that it stays in scalar registers and a
// load can take it as its scalar base next to a 32-bit lane offset.
__device__ __forceinline__ const uint8_t* uniform_ptr(const uint8_t* p) {
    const unsigned long long u = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u), hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
    return reinterpret_cast<const uint8_t*>(((unsigned long long)hi << 32) | lo);
}
// LDS transpose read: within each 16 lanes, lane j passes the address of 4 consecutive 16-bit elements
// D[j][0..3] and receives D[j/4 + 4i][j%4], i = 0..3
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x2 lds_read_tr16(unsigned lds_addr) {
    const short4v r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(size_t)lds_addr);
    return __builtin_bit_cast(u32x2, r);
}
__device__ __forceinline__ u32x4 lds_read_b128(unsigned lds_addr) {
    return *(__attribute__((address_space(3))) const u32x4*)(size_t)lds_addr;
}
__device__ __forceinline__ unsigned lds_address(const uint8_t* p) {     // byte address inside the workgroup's LDS
    return (unsigned)(size_t)(__attribute__((address_space(3))) const uint8_t*)p;
}

// Maximum over the four lanes m16, m16+16, m16+32, m16+48 (the lanes that share a query row), left in
// all four: gfx950's row and half-wave swaps stay on the vector ALU, where a shuffle goes through the
// LDS crossbar.  permlane16_swap(x, x) returns (rows 0,0,2,2 ; rows 1,1,3,3) of x, permlane32_swap(x, x)
// (lower half twice ; upper half twice).
__device__ __forceinline__ float max_over_lane_groups(float x) {
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// four E4M3 codes -> four bf16 (exact: three mantissa bits fit, the exponent range is inside bf16's)
__device__ __forceinline__ u32x2 e4m3x4_to_bf16(unsigned w) {
    const float2v a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    return u32x2{__builtin_amdgcn_perm(__float_as_uint(a[1]), __float_as_uint(a[0]), 0x07060302u),   // upper halves of both floats
                 __builtin_amdgcn_perm(__float_as_uint(b[1]), __float_as_uint(b[0]), 0x07060302u)};
}
// sixteen codes -> two 16-byte slots of bf16
__device__ __forceinline__ void e4m3x16_to_bf16(const u32x4& c, u32x4& s0, u32x4& s1) {
    const u32x2 a = e4m3x4_to_bf16(c[0]), b = e4m3x4_to_bf16(c[1]), d = e4m3x4_to_bf16(c[2]), e = e4m3x4_to_bf16(c[3]);
    s0 = u32x4{a[0], a[1], b[0], b[1]};
    s1 = u32x4{d[0], d[1], e[0], e[1]};
}

// KV8: the prefix keys/values are 8-bit E4M3 codes with one scale per KV head (the tree's own keys and
// values stay bf16).  Codes are widened to bf16 on their way into LDS; the key scale joins the softmax
// scale, the value scale multiplies the chunk's partial output.
template <int DH, int RBW, bool KV8>
__global__ __launch_bounds__(TA_THREADS, 2)
void tree_attn_bf16_kernel(const uint16_t* __restrict__ Q, const void* __restrict__ Kp, const void* __restrict__ Vp,
                           const float* __restrict__ k_scale, const float* __restrict__ v_scale,
                           const long long* __restrict__ kv_offsets, const int* __restrict__ kv_len,
                           const uint16_t* __restrict__ Kt,
                           const uint16_t* __restrict__ Vt, const unsigned long long* __restrict__ mask_bits,
                           int B, int N, int q0, int nq, int Hq, int Hkv, int chunk, int words, int nmblk, int rows_pad,
                           float scale_log2e, uint16_t* __restrict__ part_o, float* __restrict__ part_ml) {
    // RBW 16-row query blocks per wave.  One block (narrow): query fragments in registers, two tiles
    // of K/V in flight in registers, staged through one LDS tile.  Two blocks (wide; every K/V fragment
    // feeds two MFMAs and a tile is fetched once per 128 rows; pays when a KV head has more than 256
    // query rows):
    //  - bf16 prefix (DIRECT): the K/V tiles go straight from global memory into LDS -- no staging
    //    registers and no LDS writes by the waves, two LDS tiles per tensor used alternately, one barrier
    //    per tile, query fragments in registers;
    //  - 8-bit prefix: codes are widened on their way through registers into a single LDS tile; to fit two
    //    resident waves per SIMD the query fragments are parked in LDS and one tile is in flight.
    constexpr int SLOTS = DH / 8;                  // 16-byte slots per K row
    constexpr int BM = 64 * RBW;                   // query rows per workgroup
    constexpr bool DIRECT = RBW == 2 && !KV8;
    constexpr int TILE_BYTES = TA_KEYS * DH * 2;
    constexpr int NBUF = DIRECT ? 2 : 1;
    // wide 8-bit variant: the query fragments live in LDS (row-major, slots swizzled like K) instead of registers
    constexpr int Q_BYTES = (RBW == 2 && !DIRECT) ? BM * DH * 2 : 0;
    __shared__ __align__(1024) uint8_t s_all[2 * NBUF * TILE_BYTES + Q_BYTES];   // (fragment addresses are formed with xor: tiles must start on a multiple of 256)
    uint8_t* const s_k = s_all;
    uint8_t* const s_v = s_all + NBUF * TILE_BYTES;
    uint8_t* const s_q = s_all + 2 * NBUF * TILE_BYTES;

    SeqChunk sc;
    // Workgroups start in linear order (x fastest) and are dealt round-robin to the 8 XCDs.  The
    // linear id is re-cut as (chunk, row block, kv head) with the head fastest, so that the
    // workgroups running at the same time read whole contiguous key rows (all heads of the same
    // tokens) and the row blocks of one head, which re-read the same keys, start together on one
    // XCD's L2 (when the head count is a multiple of 8).
    const unsigned lin = blockIdx.x + gridDim.x * blockIdx.y;
    // (chunks are handed out last first: a sequence's short chunks -- the tree chunk and the partly filled
    // last prefix chunk -- start first and give their places to the workgroups beyond the first resident round)
    const int slot = (int)(lin / gridDim.y), yy = (int)(lin - (unsigned)slot * gridDim.y);
    const int flat = (int)gridDim.x - 1 - slot;
    if (!locate_chunk(flat, B, chunk, kv_offsets, kv_len, sc)) return;
    const int mblk = yy / Hkv, kvh = yy - mblk * Hkv;
    const int grp = Hq / Hkv, rows = grp * nq;      // query rows: tree rows q0 .. q0+nq-1 of every head in the group
    // A workgroup runs up to two phases over the same accumulators: its chunk of prefix keys (all
    // visible; 8-bit codes in the KV8 kernels), then, in a sequence's last chunk, the N tree keys under
    // the ancestor mask.  The variables below describe the phase in progress.
    const bool has_tree = sc.c == sc.nc - 1;
    const long long left = sc.P - (long long)sc.c * chunk;
    const int count_p = left <= 0 ? 0 : (left < chunk ? (int)left : chunk);
    constexpr int SLOTS_ = DH / 8;
    bool is_tree = false, codes = false;
    int count = 0, ntile = 0, spr = SLOTS_;
    size_t kv_stride = 0, kpiece = 0, tile_step = 0;
    const uint8_t *kptr = nullptr, *vptr = nullptr;   // DIRECT: uniform pointers to the next tile to fetch
    unsigned koff = 0, voff = 0;                      // DIRECT: this lane's byte offset inside a tile
    float sl2 = scale_log2e, inv_sl2 = 0.f;        // softmax scale of the phase (times the key scale for codes) and its reciprocal
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);   // (wave-uniform: a scalar)
    const int m16 = lane & 15, g4 = lane >> 4;
    // this lane's byte offsets inside a staged K / V tile for fragment step 0 (see k_frag and v_frag)
    const unsigned klane = m16 * (DH * 2) + ((g4 ^ k_swz<DH>(m16)) << 4);
    const unsigned vlane = (4 * g4 + (m16 >> 2)) * (DH * 2) + ((v_swz<DH>(4 * g4 + (m16 >> 2)) << 5) | ((m16 & 3) << 3));
    // The reference value the exp2 arguments are taken against (m_run, or 0 while the row has seen no
    // key; c_raw: the same in units of the phase's raw scores); it follows the running maximum only when a
    // score gets REF_SLACK above it.
    float m_eff[RBW], c_raw[RBW];
    constexpr float REF_SLACK = 8.f;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) { m_eff[rb] = 0.f; c_raw[rb] = 0.f; }
    auto set_phase = [&](int phase) {
        is_tree = phase == 1;
        count = is_tree ? N : count_p;
        codes = KV8 && !is_tree;
        const size_t esz = codes ? 1 : 2;
        kv_stride = (size_t)Hkv * DH * esz;            // bytes between consecutive keys
        const size_t first_key = is_tree ? (size_t)sc.b * N : (size_t)(sc.off + (long long)sc.c * chunk);
        const uint8_t* kbase = reinterpret_cast<const uint8_t*>(is_tree ? (const void*)Kt : Kp) + (first_key * Hkv + kvh) * DH * esz;
        const uint8_t* vbase = reinterpret_cast<const uint8_t*>(is_tree ? (const void*)Vt : Vp) + (first_key * Hkv + kvh) * DH * esz;
        sl2 = scale_log2e;
        if constexpr (KV8) { if (codes) sl2 *= k_scale[kvh]; }
        inv_sl2 = sl2 > 0.f ? 1.f / sl2 : 0.f;         // (a key scale of 0 -- an all-zero head -- leaves every score at 0)
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) c_raw[rb] = m_eff[rb] * inv_sl2;     // the raw unit changes with the phase's scale
        // per-thread source pointers of the next tile to fetch, advanced by one tile per fetch (no 64-bit
        // multiplies in the loop); piece i of a thread is (TA_THREADS / spr) keys after piece i-1
        spr = codes ? SLOTS_ / 2 : SLOTS_;             // 16-byte pieces per key row in memory
        kptr = kbase + (size_t)(tid / spr) * kv_stride + (tid % spr) * 16;
        vptr = vbase + (size_t)(tid / spr) * kv_stride + (tid % spr) * 16;
        if constexpr (DIRECT) {
            // A wave's load instruction fills 1 KB of LDS, lane l the 16 bytes at 16 l: lane (r, p) = (l / SLOTS,
            // l % SLOTS) owns position p of a key row and fetches the source slot the swizzle puts there.
            // The row's swizzle depends on the key index modulo 16 (8, 4) only, so it is the same for all of a
            // lane's rows, which are 4 * RPI keys apart.
            constexpr int RPI = 64 / SLOTS_;
            const int lr = w * RPI + lane / SLOTS_, pos = lane % SLOTS_;
            const int ck = pos ^ k_swz<DH>(lr), cv = (((pos >> 1) ^ v_swz<DH>(lr)) << 1) | (pos & 1);
            // addresses are a wave-uniform tile pointer (scalar registers) plus a 32-bit lane offset
            koff = (unsigned)lr * (unsigned)kv_stride + ck * 16;
            voff = (unsigned)lr * (unsigned)kv_stride + cv * 16;
            kptr = kbase;
            vptr = vbase;
        }
        kpiece = (size_t)(TA_THREADS / spr) * kv_stride;
        tile_step = (size_t)TA_KEYS * kv_stride;
        ntile = (count + TA_KEYS - 1) / TA_KEYS;
    };
    // query fragments: lane (m16, g4) holds, for its row, dh elements 32t + 8*g4 .. +7
    u32x4 qf[RBW][DH / 32];
    const unsigned long long* mptr[RBW];          // the row's ancestor bits (tree chunk only; read per tile, not held)
    int rho[RBW];
    // (called after the first K/V tiles have been requested, so that the two latencies overlap)
    auto load_queries = [&]() {
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        rho[rb] = mblk * BM + (w * RBW + rb) * 16 + m16;
        const bool ok = rho[rb] < rows;
        const int nr = ok ? rho[rb] / grp : 0, j = ok ? rho[rb] - nr * grp : 0, n = q0 + nr;
        const uint16_t* qrow = Q + (((size_t)sc.b * N + n) * Hq + kvh * grp + j) * DH;
#pragma unroll
        for (int t = 0; t < DH / 32; ++t)
            qf[rb][t] = ok ? *reinterpret_cast<const u32x4*>(qrow + t * 32 + g4 * 8) : u32x4{0u, 0u, 0u, 0u};
        mptr[rb] = ok ? mask_bits + ((size_t)sc.b * N + n) * words : nullptr;
        if constexpr (RBW == 2 && !DIRECT) {           // park the fragments in LDS; the same lane reads them back
#pragma unroll
            for (int t = 0; t < DH / 32; ++t)
                *reinterpret_cast<u32x4*>(s_q + ((w * RBW + rb) * 16 + m16) * (DH * 2) + (((t * 4 + g4) ^ k_swz<DH>((w * RBW + rb) * 16 + m16)) << 4)) = qf[rb][t];
        }
    }
    };

    floatx4 acc[RBW][DH / 16];
    floatx4 accl[RBW];                            // element 0 of lanes g4 == 0: the row's running sum of P
    float m_run[RBW];
    // A operand whose row 0 is all ones (bf16 1.0 = 0x3f80) and whose other rows are zero
    const unsigned one2 = m16 == 0 ? 0x3f803f80u : 0u;
    const u32x4 ones_row = {one2, one2, one2, one2};
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        m_run[rb] = NEG_BIG;
        accl[rb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int db = 0; db < DH / 16; ++db) acc[rb][db] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // The next tiles' K and V are fetched into registers while the current tile is multiplied.
    constexpr int NKP = TA_KEYS * SLOTS / TA_THREADS;          // 16-byte pieces of a bf16 K tile per thread
    // Two register sets.  bf16 kernels: a set holds a whole tile; the narrow variant uses both alternately
    // (tiles t+1 and t+2 in flight while tile t is multiplied), the wide one has registers for one.  8-bit
    // kernels: a set is half as large, which is a whole tile of codes (two tiles in flight in both variants);
    // their bf16 tree chunk spreads each tile over both sets.
    constexpr int NH = KV8 ? NKP / 2 : NKP;            // pieces per register set
    constexpr int DEPTH = RBW == 1 ? 2 : 1;            // bf16 kernels: tiles in flight
    u32x4 krA[NH], vrA[NH], krB[NH], vrB[NH];
    auto advance = [&]() { kptr += tile_step; vptr += tile_step; };
    // pieces I0 .. I0+NH-1 of a bf16 tile
    auto fetch_bf16 = [&](int tile, auto i0c, u32x4 (&kr)[NH], u32x4 (&vr)[NH]) {
        constexpr int I0 = decltype(i0c)::value;
        const int key0 = tile * TA_KEYS;
        if (key0 + TA_KEYS <= count) {                 // full tile (uniform): no bounds checks
#pragma unroll
            for (int i = 0; i < NH; ++i) kr[i] = *reinterpret_cast<const u32x4*>(kptr + (I0 + i) * kpiece);
#pragma unroll
            for (int i = 0; i < NH; ++i) vr[i] = *reinterpret_cast<const u32x4*>(vptr + (I0 + i) * kpiece);
        } else {
#pragma unroll
            for (int i = 0; i < NH; ++i) {
                const bool in = key0 + (tid + (I0 + i) * TA_THREADS) / SLOTS < count;
                kr[i] = in ? *reinterpret_cast<const u32x4*>(kptr + (I0 + i) * kpiece) : u32x4{0u, 0u, 0u, 0u};
                vr[i] = in ? *reinterpret_cast<const u32x4*>(vptr + (I0 + i) * kpiece) : u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    auto stage_bf16 = [&](auto i0c, const u32x4 (&kr)[NH], const u32x4 (&vr)[NH]) {
        constexpr int I0 = decltype(i0c)::value;
        // K tile -> LDS, row-major, 16-byte slots swizzled by the row
#pragma unroll
        for (int i = 0; i < NH; ++i) {
            const int p = tid + (I0 + i) * TA_THREADS, key = p / SLOTS, c = p - key * SLOTS;
            *reinterpret_cast<u32x4*>(s_k + key * (DH * 2) + ((c ^ k_swz<DH>(key)) << 4)) = kr[i];
        }
        // V tile -> LDS, row-major as well (the PV operand is transposed by the LDS read itself)
#pragma unroll
        for (int i = 0; i < NH; ++i) {
            const int p = tid + (I0 + i) * TA_THREADS, key = p / SLOTS, c = p - key * SLOTS;
            *reinterpret_cast<u32x4*>(s_v + key * (DH * 2) + ((((c >> 1) ^ v_swz<DH>(key)) << 5) | ((c & 1) << 4))) = vr[i];
        }
    };
    // DIRECT: tile -> LDS buffer `buf` without passing through registers.  Keys beyond the phase's count
    // re-read its last key (their scores are masked; a finite value keeps 0 * v finite).
    auto issue_direct = [&](int tile, int buf) {
        constexpr int RPI = 64 / SLOTS, KSTEP = 4 * RPI, NI = TA_KEYS / KSTEP;
        typedef __attribute__((address_space(1))) const void* gptr;
        typedef __attribute__((address_space(3))) void* lptr;
        const int key0 = tile * TA_KEYS;
        uint8_t* dk = s_k + buf * TILE_BYTES + w * 1024;
        uint8_t* dv = s_v + buf * TILE_BYTES + w * 1024;
        if (key0 + TA_KEYS <= count) {                 // full tile (uniform)
#pragma unroll
            for (int i = 0; i < NI; ++i)
                __builtin_amdgcn_global_load_lds((gptr)(uniform_ptr(kptr + (size_t)i * KSTEP * kv_stride) + koff), (lptr)(dk + i * 4096), 16, 0, 0);
#pragma unroll
            for (int i = 0; i < NI; ++i)
                __builtin_amdgcn_global_load_lds((gptr)(uniform_ptr(vptr + (size_t)i * KSTEP * kv_stride) + voff), (lptr)(dv + i * 4096), 16, 0, 0);
        } else {
            const int lr = w * RPI + lane / SLOTS, lim = count - 1 - key0;   // lim >= 0: the tile has a key
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int keyi = i * KSTEP + lr;
                const unsigned d = (unsigned)((keyi <= lim ? keyi : lim) - lr) * (unsigned)kv_stride;   // (wraps; koff + d >= 0)
                __builtin_amdgcn_global_load_lds((gptr)(uniform_ptr(kptr) + (koff + d)), (lptr)(dk + i * 4096), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((gptr)(uniform_ptr(vptr) + (voff + d)), (lptr)(dv + i * 4096), 16, 0, 0);
            }
        }
        advance();
    };
    // a tile of codes: NKP / 2 pieces of 16 codes per thread
    auto fetch_codes = [&](int tile, u32x4 (&kr)[NH], u32x4 (&vr)[NH]) {
        const int key0 = tile * TA_KEYS;
        if (key0 + TA_KEYS <= count) {
#pragma unroll
            for (int i = 0; i < NKP / 2; ++i) kr[i] = *reinterpret_cast<const u32x4*>(kptr + i * kpiece);
#pragma unroll
            for (int i = 0; i < NKP / 2; ++i) vr[i] = *reinterpret_cast<const u32x4*>(vptr + i * kpiece);
        } else {
#pragma unroll
            for (int i = 0; i < NKP / 2; ++i) {
                const bool in = key0 + (tid + i * TA_THREADS) / (SLOTS / 2) < count;
                kr[i] = in ? *reinterpret_cast<const u32x4*>(kptr + i * kpiece) : u32x4{0u, 0u, 0u, 0u};
                vr[i] = in ? *reinterpret_cast<const u32x4*>(vptr + i * kpiece) : u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    // a piece of 16 codes becomes the two 16-byte slots 2*c8 and 2*c8+1 of its row
    auto stage_codes = [&](const u32x4 (&kr)[NH], const u32x4 (&vr)[NH]) {
#pragma unroll
        for (int i = 0; i < NKP / 2; ++i) {
            const int p = tid + i * TA_THREADS, key = p / (SLOTS / 2), c8 = p - key * (SLOTS / 2);
            u32x4 k0, k1, v0, v1;
            e4m3x16_to_bf16(kr[i], k0, k1);
            e4m3x16_to_bf16(vr[i], v0, v1);
            *reinterpret_cast<u32x4*>(s_k + key * (DH * 2) + (((2 * c8) ^ k_swz<DH>(key)) << 4)) = k0;
            *reinterpret_cast<u32x4*>(s_k + key * (DH * 2) + (((2 * c8 + 1) ^ k_swz<DH>(key)) << 4)) = k1;
            *reinterpret_cast<u32x4*>(s_v + key * (DH * 2) + ((c8 ^ v_swz<DH>(key)) << 5)) = v0;
            *reinterpret_cast<u32x4*>(s_v + key * (DH * 2) + (((c8 ^ v_swz<DH>(key)) << 5) | 16)) = v1;
        }
    };
    // the tile staged in LDS (keys tile*64 ..) against the query fragments
    auto compute = [&](int tile, int buf = 0) {
        const int key0 = tile * TA_KEYS;
        const uint8_t* const sk = s_k + buf * TILE_BYTES;
        const uint8_t* const sv_ = s_v + buf * TILE_BYTES;
        constexpr int KBH = TA_KEYS / 16;              // 16-key blocks of the tile
        // S^T = K Q^T : s[rb][kq][i] = score(query row of this lane, key kq*16 + 4*g4 + i)
        // (the accumulators start at minus the row's reference value, in units of raw scores)
        floatx4 s[RBW][KBH];
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
            for (int kq = 0; kq < KBH; ++kq) s[rb][kq] = floatx4{-c_raw[rb], -c_raw[rb], -c_raw[rb], -c_raw[rb]};
        // K fragment (step t, key block kq): row kq*16 + m16, slot (4t + g4) ^ swizzle.  The swizzle is the
        // same for all of a lane's rows and 4t + g4 = 4t ^ g4, so the address is one lane constant with
        // t << 6 xor-ed in and the key block as an immediate offset.
        const unsigned kl = lds_address(sk) + klane;
        auto k_frag = [&](int t, int kq) -> u32x4 { return lds_read_b128((kl ^ (unsigned)(t << 6)) + kq * 16 * (DH * 2)); };
        if constexpr (DIRECT) {
            // the K fragments of step t+1 are read from LDS while step t is multiplied (two register sets)
            u32x4 kf[2][KBH];
#pragma unroll
            for (int kq = 0; kq < KBH; ++kq) kf[0][kq] = k_frag(0, kq);
            __builtin_amdgcn_sched_group_barrier(0x100, KBH, 0);
#pragma unroll
            for (int t = 0; t < DH / 32; ++t) {
#pragma unroll
                for (int kq = 0; kq < KBH; ++kq) {
                    if (t + 1 < DH / 32) kf[(t + 1) & 1][kq] = k_frag(t + 1, kq);
#pragma unroll
                    for (int rb = 0; rb < RBW; ++rb)
                        s[rb][kq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, kf[t & 1][kq]), __builtin_bit_cast(bf16x8, qf[rb][t]), s[rb][kq], 0, 0, 0);
                    if (t + 1 < DH / 32) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read ...
                    __builtin_amdgcn_sched_group_barrier(0x008, RBW, 0);                        // ... then the block's MFMAs
                }
            }
        } else {
#pragma unroll
        for (int t = 0; t < DH / 32; ++t) {            // t outside: consecutive MFMAs go to different accumulators
            u32x4 qv[RBW];
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
                if constexpr (RBW == 2)
                    qv[rb] = *reinterpret_cast<const u32x4*>(s_q + ((w * RBW + rb) * 16 + m16) * (DH * 2) + (((t * 4 + g4) ^ k_swz<DH>((w * RBW + rb) * 16 + m16)) << 4));
                else
                    qv[rb] = qf[rb][t];
            }
#pragma unroll
            for (int kq = 0; kq < KBH; ++kq) {
                const u32x4 kf = k_frag(t, kq);
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
                    s[rb][kq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, kf), __builtin_bit_cast(bf16x8, qv[rb]), s[rb][kq], 0, 0, 0);
            }
        }
        }

        bf16x8 pf[RBW][KBH / 2];
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
            // s holds raw score - c_raw, c_raw = the row's reference in raw units.  While no score of the wave
            // climbs more than REF_SLACK (after scaling) above its row's reference (and every row has one) the
            // probabilities are exp2(s * scale): no maximum across lanes, no rescaling.  They may then
            // exceed 1 (by at most 2^REF_SLACK), which float32 sums and bf16 products carry without loss.
            float mx = s[rb][0][0];
#pragma unroll
            for (int kq = 0; kq < KBH; ++kq)
#pragma unroll
                for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[rb][kq][i]);
            const bool plain = !is_tree && key0 + TA_KEYS <= count;     // uniform: every key of the tile is visible
            if (plain && !__any(mx * sl2 > REF_SLACK || m_run[rb] <= NEG_BIG)) {
#pragma unroll
                for (int kq = 0; kq < KBH; ++kq)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        pf[rb][kq >> 1][(kq & 1) * 4 + i] = (__bf16)__builtin_amdgcn_exp2f(s[rb][kq][i] * sl2);
            } else {
                // new reference: the row's running maximum (scaled scores = s * scale + m_eff)
                const unsigned long long mword = (is_tree && mptr[rb] != nullptr && (key0 >> 6) < words) ? mptr[rb][key0 >> 6] : 0ull;
                floatx4 sm[KBH];
                float mt = -INFINITY;
#pragma unroll
                for (int kq = 0; kq < KBH; ++kq) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int key = key0 + kq * 16 + g4 * 4 + i;
                        bool vis = key < count;
                        if (is_tree) vis = vis && ((mword >> (key & 63)) & 1ull);
                        const float v = vis ? __builtin_fmaf(s[rb][kq][i], sl2, m_eff[rb]) : -INFINITY;
                        sm[kq][i] = v;
                        mt = fmaxf(mt, v);
                    }
                }
                mt = max_over_lane_groups(mt);
                const float m_new = fmaxf(m_run[rb], mt);      // stays NEG_BIG while the row has seen no key
                const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_new);
                m_run[rb] = m_new;
                m_eff[rb] = m_new <= NEG_BIG ? 0.f : m_new;
                c_raw[rb] = m_eff[rb] * inv_sl2;
#pragma unroll
                for (int kq = 0; kq < KBH; ++kq)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        pf[rb][kq >> 1][(kq & 1) * 4 + i] = (__bf16)__builtin_amdgcn_exp2f(sm[kq][i] - m_new);
#pragma unroll
                for (int db = 0; db < DH / 16; ++db) acc[rb][db] *= alpha;
                accl[rb] *= alpha;
            }
        }

        // O^T += V^T P^T : keys of MFMA u for lane group g4 are {32u + 4g4 + i} and {32u + 16 + 4g4 + i}
        const unsigned vl = lds_address(sv_) + vlane;
        auto v_frag = [&](int db, int uq) -> u32x4 {
            const int u = uq;
            // lane (m16, g4) passes key row 32u (+16) + 4*g4 + m16/4, dh db*16 + 4*(m16%4) .. +3 and
            // receives dh db*16 + m16 of keys 32u (+16) + 4*g4 + i
            // (the granule swizzle depends on the key modulo 8 (4) only: one lane constant with db << 5 xor-ed
            // in, the key block as an immediate offset)
            const unsigned a = (vl ^ (unsigned)(db << 5)) + 32 * u * (DH * 2);
            const u32x2 va = lds_read_tr16(a), vb = lds_read_tr16(a + 16 * (DH * 2));
            return u32x4{va[0], va[1], vb[0], vb[1]};
        };
        if constexpr (DIRECT) {
            // the V fragments of block db+1 are read from LDS while block db is multiplied
            u32x4 vf[2][KBH / 2];
#pragma unroll
            for (int uq = 0; uq < KBH / 2; ++uq) vf[0][uq] = v_frag(0, uq);
            __builtin_amdgcn_sched_group_barrier(0x100, KBH, 0);
#pragma unroll
            for (int db = 0; db < DH / 16; ++db) {
#pragma unroll
                for (int uq = 0; uq < KBH / 2; ++uq) {
                    if (db + 1 < DH / 16) vf[(db + 1) & 1][uq] = v_frag(db + 1, uq);
#pragma unroll
                    for (int rb = 0; rb < RBW; ++rb)
                        acc[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, vf[db & 1][uq]), pf[rb][uq], acc[rb][db], 0, 0, 0);
                    if (db + 1 < DH / 16) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, RBW, 0);
                }
            }
        } else {
#pragma unroll
        for (int db = 0; db < DH / 16; ++db) {
#pragma unroll
            for (int uq = 0; uq < KBH / 2; ++uq) {
                const u32x4 vf = v_frag(db, uq);
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
                    acc[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, vf), pf[rb][uq], acc[rb][db], 0, 0, 0);
            }
        }
        }
        // the row sums of P come out of the same product with a row of ones in place of a V^T row: the
        // normaliser is the sum of exactly the rounded probabilities the numerator used
#pragma unroll
        for (int uq = 0; uq < KBH / 2; ++uq)
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
                accl[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ones_row), pf[rb][uq], accl[rb], 0, 0, 0);
    };
    using std::integral_constant;
    bool q_loaded = false;
    int bufi = 0;                                      // DIRECT: LDS tile the next first fetch of a phase goes to
#pragma unroll
    for (int phase = 0; phase < 2; ++phase) {
        if (phase == 0 ? count_p == 0 : !has_tree) continue;
        set_phase(phase);
        if (KV8 && codes) {
            if constexpr (KV8) {
                if (ntile > 0) { fetch_codes(0, krA, vrA); advance(); }
                if (ntile > 1) { fetch_codes(1, krB, vrB); advance(); }
                if (!q_loaded) { load_queries(); q_loaded = true; }
                for (int tile = 0; tile < ntile; tile += 2) {
                    __syncthreads();                       // previous tile fully consumed
                    stage_codes(krA, vrA);
                    __syncthreads();
                    if (tile + 2 < ntile) { fetch_codes(tile + 2, krA, vrA); advance(); }
                    compute(tile);
                    if (tile + 1 < ntile) {
                        __syncthreads();
                        stage_codes(krB, vrB);
                        __syncthreads();
                        if (tile + 3 < ntile) { fetch_codes(tile + 3, krB, vrB); advance(); }
                        compute(tile + 1);
                    }
                }
            }
        } else if constexpr (DIRECT) {
            // Tile t+1 is on its way into one LDS buffer while tile t is multiplied out of the other.  The
            // barrier of tile t says that every wave's part of tile t has landed and that every wave is done
            // with tile t-1, whose buffer the loads issued right after it overwrite.  A phase's first loads go
            // to the buffer the last-but-one product used, which every wave left before the last barrier.
            issue_direct(0, bufi);
            if (!q_loaded) { load_queries(); q_loaded = true; }
            for (int tile = 0; tile < ntile; ++tile) {
                __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wave's loads into LDS are complete
                __syncthreads();
                if (tile + 1 < ntile) issue_direct(tile + 1, bufi ^ 1);
                compute(tile, bufi);
                bufi ^= 1;
            }
        } else if constexpr (KV8) {                        // bf16 tree chunk of an 8-bit kernel: one tile across both sets
            if (ntile > 0) { fetch_bf16(0, integral_constant<int, 0>{}, krA, vrA); fetch_bf16(0, integral_constant<int, NH>{}, krB, vrB); advance(); }
            if (!q_loaded) { load_queries(); q_loaded = true; }
            for (int tile = 0; tile < ntile; ++tile) {
                __syncthreads();
                stage_bf16(integral_constant<int, 0>{}, krA, vrA);
                stage_bf16(integral_constant<int, NH>{}, krB, vrB);
                __syncthreads();
                if (tile + 1 < ntile) {
                    fetch_bf16(tile + 1, integral_constant<int, 0>{}, krA, vrA);
                    fetch_bf16(tile + 1, integral_constant<int, NH>{}, krB, vrB);
                    advance();
                }
                compute(tile);
            }
        } else {
            constexpr integral_constant<int, 0> z{};
            auto do_tile = [&](int tile, u32x4 (&kr)[NH], u32x4 (&vr)[NH]) {
                __syncthreads();                           // previous tile fully consumed
                stage_bf16(z, kr, vr);
                __syncthreads();
                if (tile + DEPTH < ntile) { fetch_bf16(tile + DEPTH, z, kr, vr); advance(); }
                compute(tile);
            };
            if (ntile > 0) { fetch_bf16(0, z, krA, vrA); advance(); }
            if constexpr (DEPTH == 2) {
                if (ntile > 1) { fetch_bf16(1, z, krB, vrB); advance(); }
                if (!q_loaded) { load_queries(); q_loaded = true; }
                for (int tile = 0; tile < ntile; tile += 2) {
                    do_tile(tile, krA, vrA);
                    if (tile + 1 < ntile) do_tile(tile + 1, krB, vrB);
                }
            } else {
                if (!q_loaded) { load_queries(); q_loaded = true; }
                for (int tile = 0; tile < ntile; ++tile) do_tile(tile, krA, vrA);
            }
        }

        if constexpr (KV8) {
            if (codes) {                               // the value scale of the codes, before bf16 tree values are added
                const float vs = v_scale[kvh];
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                    for (int db = 0; db < DH / 16; ++db) acc[rb][db] *= vs;
            }
        }
    }
    if (!q_loaded) load_queries();                     // (every chunk has keys; the row numbers are needed below)
    __syncthreads();                                   // every wave is done with the tiles: LDS is reused below

    // Partial results of this chunk: un-normalised O (lane holds dh db*16 + 4*g4 + i of its row), max, sum.
    // All workgroups finish together and nothing hides their stores, so O leaves as 16-bit floats: every row
    // is scaled by the power of two (exact) that puts its largest magnitude into [2^14, 2^15), rounded to
    // nearest fp16 (11 significant bits for everything within 2^-28 of the row's largest value; the output is
    // bf16, 8 bits) and the scale's inverse travels with (max, sum).
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        const float l = accl[rb][0];                // valid in the lanes that write it (g4 == 0)
        float am = 0.f;
#pragma unroll
        for (int db = 0; db < DH / 16; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) am = fmaxf(am, fabsf(acc[rb][db][i]));
        am = max_over_lane_groups(am);              // the row's largest magnitude (all lanes take part)
        unsigned eb = (__float_as_uint(am) >> 23) & 255u;        // am = 1.f x 2^(eb - 127)
        eb = eb < 16u ? 16u : eb;                   // (rows of magnitude below 2^-111 go out as zeros)
        const float up = __uint_as_float((268u - eb) << 23);     // 2^(141 - eb): am * up is in [2^14, 2^15)
        const float down = __uint_as_float((eb - 14u) << 23);    // 2^(eb - 141)
        // through a wave-private piece of LDS (the K/V tiles are done with), so that a store instruction writes whole
        // rows: lane (m16, g4) leaves 8 bytes per 16-column block in its row (rows 16 bytes apart in bank terms), and
        // takes back 16 bytes of row l / 16 (+ 4, 8, 12) at 16 (l % 16)
        constexpr int RS = DH * 2 + 16;                 // LDS row stride
        static_assert(4 * RBW * 16 * RS <= (int)sizeof(s_all), "the staging rows fit into the tile buffers");
        uint8_t* stage = s_all + (w * RBW + rb) * 16 * RS;
#pragma unroll
        for (int db = 0; db < DH / 16; ++db) {
            const _Float16 h0 = (_Float16)(acc[rb][db][0] * up), h1 = (_Float16)(acc[rb][db][1] * up);
            const _Float16 h2 = (_Float16)(acc[rb][db][2] * up), h3 = (_Float16)(acc[rb][db][3] * up);
            u32x2 pk;
            pk[0] = (unsigned)__builtin_bit_cast(uint16_t, h0) | ((unsigned)__builtin_bit_cast(uint16_t, h1) << 16);
            pk[1] = (unsigned)__builtin_bit_cast(uint16_t, h2) | ((unsigned)__builtin_bit_cast(uint16_t, h3) << 16);
            *reinterpret_cast<u32x2*>(stage + m16 * RS + (db * 16 + g4 * 4) * 2) = pk;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const int rho0 = mblk * BM + (w * RBW + rb) * 16;      // first row of the block
        constexpr int CPR = DH * 2 / 16;                       // 16-byte pieces per row
#pragma unroll
        for (int k2 = 0; k2 < 16 * CPR / 64; ++k2) {
            const int rr = (k2 * 64 + lane) / CPR, cc = (k2 * 64 + lane) % CPR;
            const u32x4 piece = *reinterpret_cast<const u32x4*>(stage + rr * RS + cc * 16);
            if (rho0 + rr < rows) {
                const size_t prow = ((size_t)flat * Hkv + kvh) * rows_pad + rho0 + rr;
                // (streaming stores: whole lines go out while other workgroups still multiply, instead of waiting
                // in L2 for the write-back at the end of the kernel)
                __builtin_nontemporal_store(piece, reinterpret_cast<u32x4*>(part_o + prow * DH + cc * 8));
            }
        }
        if (rho[rb] < rows && g4 == 0) {
            const size_t prow = ((size_t)flat * Hkv + kvh) * rows_pad + rho[rb];
            part_ml[prow * 3] = m_run[rb]; part_ml[prow * 3 + 1] = l; part_ml[prow * 3 + 2] = down;
        }
    }
}

// grid (B*N, Hq / 4), 4 waves: one wave per (row, head).  Lanes first act as chunks (max and
// weights of up to 64 chunks at a time), then as DH / 64 consecutive dh columns each for the weighted
// sum of the 16-bit partial outputs (a wave reads a partial row as one contiguous piece), whose loads
// are independent and issued eight chunks at a time.
template <int DH>
__global__ __launch_bounds__(256)
void tree_attn_combine_kernel(const long long* __restrict__ kv_offsets, const int* __restrict__ kv_len, int N, int q0, int nq, int Hq, int Hkv, int chunk, int rows_pad,
                              int max_chunks, const uint16_t* __restrict__ part_o, const float* __restrict__ part_ml,
                              uint16_t* __restrict__ O, float* __restrict__ lse) {
    const int b = blockIdx.x / nq, nr = blockIdx.x - b * nq, n = q0 + nr, bn = b * N + n;
    const int h = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (h >= Hq) return;
    const int grp = Hq / Hkv, kvh = h / grp, rho = nr * grp + (h - kvh * grp);
    int first, nc;
    locate_seq(b, chunk, kv_offsets, kv_len, first, nc);
    // the split-KV kernel ran max_chunks chunks (sized from the host's total_prefix); if the device offsets
    // describe more, the excess was never computed and must not be read
    if (first > max_chunks) first = max_chunks;
    if (first + nc > max_chunks) nc = max_chunks - first;
    const size_t cstride = (size_t)Hkv * rows_pad;               // rows between consecutive chunks
    const size_t row0 = ((size_t)first * Hkv + kvh) * rows_pad + rho;
    float mx = NEG_BIG;
    for (int c = lane; c < nc; c += 64) mx = fmaxf(mx, part_ml[(row0 + c * cstride) * 3]);
    mx = wave_max(mx);
    float l = 0.f, o[DH / 64];
#pragma unroll
    for (int e = 0; e < DH / 64; ++e) o[e] = 0.f;
    for (int c0 = 0; c0 < nc; c0 += 64) {
        const int c = c0 + lane;
        float wgt = 0.f, lc = 0.f, wo = 0.f;           // wo: the chunk's weight times the scale of its 16-bit values
        if (c < nc) {
            wgt = exp2f(part_ml[(row0 + c * cstride) * 3] - mx);
            lc = part_ml[(row0 + c * cstride) * 3 + 1];
            wo = wgt * part_ml[(row0 + c * cstride) * 3 + 2];
        }
        l += wave_sumf(wgt * lc);
        const int nb = min(64, nc - c0);
        constexpr int CU = 8;                          // partial outputs in flight per lane
        for (int j = 0; j < nb; j += CU) {             // (the last group may be short: its loads are skipped, not serialised)
            // (a short last group re-reads its last chunk with weight 0: no branches, the loads stay independent)
            unsigned v[CU];
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const int cu = min(j + u, nb - 1);
                const uint16_t* src = part_o + (row0 + (size_t)(c0 + cu) * cstride) * DH + lane * (DH / 64);
                if constexpr (DH == 128) v[u] = *reinterpret_cast<const unsigned*>(src);
                else v[u] = src[0];
            }
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const float wu = j + u < nb ? read_lane_dyn(wo, j + u) : 0.f;
#pragma unroll
                for (int e = 0; e < DH / 64; ++e) o[e] += wu * (float)__builtin_bit_cast(_Float16, (uint16_t)(v[u] >> (16 * e)));
            }
        }
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    uint16_t* orow = O + ((size_t)bn * Hq + h) * DH + lane * (DH / 64);   // this lane's columns
    if constexpr (DH == 128) {
        const __bf16 v0 = (__bf16)(o[0] * inv), v1 = (__bf16)(o[1] * inv);
        *reinterpret_cast<unsigned*>(orow) = (unsigned)__builtin_bit_cast(uint16_t, v0) | ((unsigned)__builtin_bit_cast(uint16_t, v1) << 16);
    } else {
        const __bf16 v0 = (__bf16)(o[0] * inv);
        orow[0] = __builtin_bit_cast(uint16_t, v0);
    }
    if (lse != nullptr && lane == 0) lse[(size_t)bn * Hq + h] = (mx + log2f(l)) * 0.6931471805599453f;
}

// fp32: one workgroup per (sequence, row, head); waves stride over keys, lanes over dh
template <int DH>
__global__ __launch_bounds__(256)
void tree_attn_f32_kernel(const float* __restrict__ Q, const float* __restrict__ Kp, const float* __restrict__ Vp,
                          const long long* __restrict__ kv_offsets, const int* __restrict__ kv_len,
                          const float* __restrict__ Kt,
                          const float* __restrict__ Vt, const unsigned long long* __restrict__ mask_bits,
                          int N, int q0, int nq, int Hq, int Hkv, int words, float scale, float* __restrict__ O, float* __restrict__ lse) {
    constexpr int E = DH / 64;
    const int h = blockIdx.x % Hq, bq = blockIdx.x / Hq, b = bq / nq, bn = b * N + q0 + (bq - b * nq);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int kvh = h / (Hq / Hkv);
    const long long off = kv_offsets[b];
    const int P = (int)prefix_keys(b, kv_offsets, kv_len);
    float q[E], o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) { q[e] = Q[((size_t)bn * Hq + h) * DH + e * 64 + lane]; o[e] = 0.f; }
    float m = NEG_BIG, l = 0.f;
    const unsigned long long* mb = mask_bits + (size_t)bn * words;
    for (int key = w; key < P + N; key += 4) {
        const float* kr; const float* vr;
        if (key < P) {
            kr = Kp + ((size_t)(off + key) * Hkv + kvh) * DH;
            vr = Vp + ((size_t)(off + key) * Hkv + kvh) * DH;
        } else {
            const int j = key - P;
            if (!((mb[j >> 6] >> (j & 63)) & 1ull)) continue;
            kr = Kt + (((size_t)b * N + j) * Hkv + kvh) * DH;
            vr = Vt + (((size_t)b * N + j) * Hkv + kvh) * DH;
        }
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) d += q[e] * kr[e * 64 + lane];
#pragma unroll
        for (int x = 32; x > 0; x >>= 1) d += __shfl_xor(d, x, 64);
        const float s = d * scale;
        const float m_new = fmaxf(m, s);
        const float alpha = __expf(m - m_new), p = __expf(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = o[e] * alpha + p * vr[e * 64 + lane];
        m = m_new;
    }
    __shared__ float s_m[4], s_l[4], s_o[4][DH];
    if (lane == 0) { s_m[w] = m; s_l[w] = l; }
#pragma unroll
    for (int e = 0; e < E; ++e) s_o[w][e * 64 + lane] = o[e];
    __syncthreads();
    if (w == 0) {
        float mx = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float lt = 0.f, ot[E];
#pragma unroll
        for (int e = 0; e < E; ++e) ot[e] = 0.f;
        for (int i = 0; i < 4; ++i) {
            const float wgt = __expf(s_m[i] - mx);
            lt += wgt * s_l[i];
#pragma unroll
            for (int e = 0; e < E; ++e) ot[e] += wgt * s_o[i][e * 64 + lane];
        }
#pragma unroll
        for (int e = 0; e < E; ++e) O[((size_t)bn * Hq + h) * DH + e * 64 + lane] = ot[e] / lt;
        if (lse != nullptr && lane == 0) lse[(size_t)bn * Hq + h] = mx + __logf(lt);
    }
}

struct AttnPlan { int rbw, bm, nmblk, rows_pad, chunk, max_chunks; size_t o_bytes, total; };
static AttnPlan attn_plan(const eagle2_cfg* cfg, const eagle2_attn_cfg* a, int nq) {
    AttnPlan p;
    const int rows = a->n_q_heads / a->n_kv_heads * nq;   // nq: tree rows that act as queries
    p.rbw = rows > 256 ? 2 : 1;                        // 16-row blocks per wave: two pay only when the kernel is compute-bound
    p.bm = 64 * p.rbw;                                 // query rows per workgroup
    p.nmblk = (rows + p.bm - 1) / p.bm;
    p.rows_pad = p.nmblk * p.bm;
    // One resident round of workgroups (two per compute unit) when the prefix is short enough; at
    // least two tiles per chunk.  (A sequence's tree keys ride with its last chunk.)
    const long long wg_per_chunk = (long long)a->n_kv_heads * p.nmblk;
    const long long target = (long long)device_cu_count() * 2;
    // sum over sequences of ceil(P_b / chunk) is at most total / chunk + batch (exactly ceil for one sequence)
    long long budget = target / wg_per_chunk - (cfg->batch > 1 ? cfg->batch : 0);
    if (budget < 1) budget = 1;
    long long want = (a->total_prefix + budget - 1) / budget;
    want = (want + TA_KEYS - 1) / TA_KEYS * TA_KEYS;
    if (want < 2 * TA_KEYS) want = 2 * TA_KEYS;
    if (want > 2048) want = 2048;                      // bounded chunks keep ragged batches balanced
    p.chunk = (int)want;
    p.max_chunks = (int)(a->total_prefix / p.chunk) + cfg->batch;
    p.o_bytes = round_up((size_t)p.max_chunks * a->n_kv_heads * p.rows_pad * a->head_dim * sizeof(uint16_t), 256);
    p.total = p.o_bytes + round_up((size_t)p.max_chunks * a->n_kv_heads * p.rows_pad * 3 * sizeof(float), 256);
    return p;
}
size_t attn_workspace_rows(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int nq) {
    return cfg->dtype == EAGLE2_DTYPE_BF16 ? attn_plan(cfg, attn, nq).total : 0;
}
size_t attn_workspace(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn) {
    return cfg->dtype == EAGLE2_DTYPE_BF16 ? attn_plan(cfg, attn, cfg->n_tree).total : 0;   // a window of rows needs no more
}

// Attention of the tree rows q0 .. q0+nq-1 (queries) over the prefix and all N tree keys under the
// mask; the public entry point asks for every row, the draft model's forward for the rows of one pass.
int tree_attn_rows(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int q0, int nq,
                   const void* Q, const void* K_prefix, const void* V_prefix, const float* k_scale, const float* v_scale,
                   const int64_t* kv_offsets, const int32_t* kv_len,
                   const void* K_tree, const void* V_tree,
                   const uint64_t* mask_bits, void* O, float* lse,
                   void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    rc = validate_attn(cfg, attn);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(Q && kv_offsets && K_tree && V_tree && mask_bits && O, EAGLE2_ERR_ARG, "eagle2_tree_attn: null pointer argument");
    E2_REQUIRE(attn->total_prefix == 0 || (K_prefix && V_prefix), EAGLE2_ERR_ARG, "eagle2_tree_attn: null KV prefix");
    E2_REQUIRE(aligned16(Q) && aligned16(K_prefix) && aligned16(V_prefix) && aligned16(K_tree) && aligned16(V_tree) && aligned16(O),
               EAGLE2_ERR_ARG, "eagle2_tree_attn: tensors must be 16-byte aligned");
    const bool kv8 = k_scale != nullptr || v_scale != nullptr;
    if (kv8) {
        E2_REQUIRE(k_scale && v_scale, EAGLE2_ERR_ARG, "tree attention: 8-bit prefix needs both k_scale and v_scale");
        E2_REQUIRE(cfg->dtype == EAGLE2_DTYPE_BF16, EAGLE2_ERR_SHAPE, "tree attention: the 8-bit prefix goes with dtype bf16 only");
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = cfg->batch, N = cfg->n_tree, Hq = attn->n_q_heads, Hkv = attn->n_kv_heads, dh = attn->head_dim;
    E2_REQUIRE(q0 >= 0 && nq >= 1 && q0 + nq <= N, EAGLE2_ERR_ARG, "tree attention: query rows %d..%d outside the tree", q0, q0 + nq - 1);
    const float scale = attn->scale > 0.f ? attn->scale : 1.0f / sqrtf((float)dh);
    const int words = (N + 63) / 64;
    const long long* offs = reinterpret_cast<const long long*>(kv_offsets);
    const unsigned long long* mb = reinterpret_cast<const unsigned long long*>(mask_bits);

    if (cfg->dtype == EAGLE2_DTYPE_F32) {
        dim3 grid((unsigned)((size_t)B * nq * Hq));
        timing_begin(1, st);
        if (dh == 128)
            hipLaunchKernelGGL((tree_attn_f32_kernel<128>), grid, dim3(256), 0, st, (const float*)Q, (const float*)K_prefix,
                               (const float*)V_prefix, offs, kv_len, (const float*)K_tree, (const float*)V_tree, mb, N, q0, nq, Hq, Hkv, words,
                               scale, (float*)O, lse);
        else
            hipLaunchKernelGGL((tree_attn_f32_kernel<64>), grid, dim3(256), 0, st, (const float*)Q, (const float*)K_prefix,
                               (const float*)V_prefix, offs, kv_len, (const float*)K_tree, (const float*)V_tree, mb, N, q0, nq, Hq, Hkv, words,
                               scale, (float*)O, lse);
        timing_end(1, st);
        E2_HIP(hipGetLastError());
        return EAGLE2_OK;
    }

    const AttnPlan p = attn_plan(cfg, attn, nq);
    E2_REQUIRE(workspace && workspace_bytes >= p.total, EAGLE2_ERR_WORKSPACE,
               "eagle2_tree_attn: workspace of %zu bytes, need %zu", workspace_bytes, p.total);
    uint16_t* part_o = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(workspace));
    float* part_ml = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + p.o_bytes);
    const float sl2 = scale * 1.4426950408889634f;
    dim3 grid(p.max_chunks, Hkv * p.nmblk);
    timing_begin(1, st);
#define E2_ATTN(DHV, RB, K8)                                                                                          \
    hipLaunchKernelGGL((tree_attn_bf16_kernel<DHV, RB, K8>), grid, dim3(TA_THREADS), 0, st, (const uint16_t*)Q,        \
                       K_prefix, V_prefix, k_scale, v_scale, offs, kv_len, (const uint16_t*)K_tree,                   \
                       (const uint16_t*)V_tree, mb, B, N, q0, nq, Hq, Hkv, p.chunk, words, p.nmblk, p.rows_pad, sl2, part_o, part_ml)
#define E2_ATTN_RB(DHV, K8) do { if (p.rbw == 2) E2_ATTN(DHV, 2, K8); else E2_ATTN(DHV, 1, K8); } while (0)
    if (dh == 128) { if (kv8) E2_ATTN_RB(128, true); else E2_ATTN_RB(128, false); }
    else           { if (kv8) E2_ATTN_RB(64, true); else E2_ATTN_RB(64, false); }
#undef E2_ATTN_RB
#undef E2_ATTN
    timing_end(1, st);
    E2_HIP(hipGetLastError());
    dim3 cgrid(B * nq, (Hq + 3) / 4);
    if (dh == 128)
        hipLaunchKernelGGL((tree_attn_combine_kernel<128>), cgrid, dim3(256), 0, st, offs, kv_len, N, q0, nq, Hq, Hkv, p.chunk, p.rows_pad,
                           p.max_chunks, part_o, part_ml, (uint16_t*)O, lse);
    else
        hipLaunchKernelGGL((tree_attn_combine_kernel<64>), cgrid, dim3(256), 0, st, offs, kv_len, N, q0, nq, Hq, Hkv, p.chunk, p.rows_pad,
                           p.max_chunks, part_o, part_ml, (uint16_t*)O, lse);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_tree_attn(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn,
                                const void* Q, const void* K_prefix, const void* V_prefix,
                                const int64_t* kv_offsets, const int32_t* kv_len,
                                const void* K_tree, const void* V_tree,
                                const uint64_t* mask_bits, void* O, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream) {
    E2_REQUIRE(cfg != nullptr, EAGLE2_ERR_ARG, "cfg is null");
    return tree_attn_rows(cfg, attn, 0, cfg->n_tree, Q, K_prefix, V_prefix, nullptr, nullptr, kv_offsets, kv_len, K_tree, V_tree,
                          mask_bits, O, lse, workspace, workspace_bytes, stream);
}

extern "C" int eagle2_tree_attn_fp8kv(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn,
                                      const void* Q, const void* K_prefix8, const void* V_prefix8,
                                      const float* k_scale, const float* v_scale,
                                      const int64_t* kv_offsets, const int32_t* kv_len,
                                      const void* K_tree, const void* V_tree,
                                      const uint64_t* mask_bits, void* O, float* lse,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    E2_REQUIRE(cfg != nullptr, EAGLE2_ERR_ARG, "cfg is null");
    E2_REQUIRE(k_scale && v_scale, EAGLE2_ERR_ARG, "eagle2_tree_attn_fp8kv: null scale pointer");
    return tree_attn_rows(cfg, attn, 0, cfg->n_tree, Q, K_prefix8, V_prefix8, k_scale, v_scale, kv_offsets, kv_len, K_tree, V_tree,
                          mask_bits, O, lse, workspace, workspace_bytes, stream);
}
