// Expansion phase (Section 4.1 of the EAGLE-2 paper): draft LM-head projection of the
// frontier rows, log-softmax, per-row top-k, joint-score accumulation along the path
// (value equation of Section 4.1, as a sum of logs) and selection of the next frontier.
//
// Two kernels per pass with at most 16 frontier rows:
//   lmhead_kernel       streams W once from HBM; per workgroup and frontier row it
//                       emits a partial (max, sum-exp, top-k) over the vocab rows it saw
//   expand_merge_kernel merges the partials, appends the k children per row with their
//                       joint scores and picks the next frontier
// With more rows (batched serving) there are two other kernels:
//   lmhead_gemm128_kernel (bf16) / lmhead_gemm_kernel (float32, after pack_h_kernel has re-tiled
//                       the frontier rows into MFMA fragment order)  stream W once per 160 rows
//                       and write the raw logits
//   row_expand_kernel   one workgroup per row: the row's (max, sum-exp, top-k) and then the
//                       same merge, children and frontier selection
//
// lmhead_kernel layout.  The contraction runs on the matrix cores with the *weight tile*
// as the 16-row A operand and the (zero-padded to 16) frontier rows as the B operand, so
// an output register holds (vocab row 4g+i, frontier row lane%16): every lane owns one
// frontier row and all per-row statistics stay in registers.  A workgroup (4 waves)
// owns tasks of 64 vocab rows; wave w streams byte range [w*RB/4, (w+1)*RB/4) of those
// rows (split-K inside the workgroup), 256 bytes per row per stage, with quarter-wave
// coalesced 16-byte loads that are staged through LDS into MFMA fragment order.  The
// next stage's loads are in flight while the current stage is multiplied.

#include "common.h"
#include <type_traits>

namespace eagle2 {

constexpr int LM_THREADS = 256;
constexpr int LM_ROWS = 64;                  // vocab rows per task
constexpr int LM_CHUNK = 256;                // bytes per row per stage per wave
constexpr int LM_RS = LM_CHUNK;              // LDS row stride; 16-byte slots are XOR-swizzled by the row
constexpr int LM_STAGE = LM_ROWS * LM_RS;    // bytes of LDS per wave (4 waves: 64 KB)
constexpr int LM_LOADS = LM_ROWS * LM_CHUNK / 1024;   // 16-byte loads per lane per stage
constexpr int LM_GMAX = 1024;                // upper bound on workgroups (partials per row)

// Orders are turned into single unsigned 64-bit comparisons.  (value, id) with "higher value first,
// then lower id": the float's bits mapped monotonically to an unsigned, above the complemented id.
__device__ __forceinline__ unsigned long long order_key(float v, int id) {
    const unsigned b = __float_as_uint(v + 0.f);       // -0 and +0 are one value
    const unsigned u = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
    return ((unsigned long long)u << 32) | (unsigned)~id;
}
__device__ __forceinline__ unsigned long long order_key(double v) {      // ties are broken by position
    const unsigned long long b = (unsigned long long)__double_as_longlong(v + 0.0);
    return b ^ ((b >> 63) ? ~0ull : 0x8000000000000000ull);
}
__device__ __forceinline__ float key_value(unsigned long long key) {
    const unsigned u = (unsigned)(key >> 32);
    return __uint_as_float(u ^ ((u >> 31) ? 0x80000000u : 0xffffffffu));
}
__device__ __forceinline__ int key_id(unsigned long long key) { return (int)~(unsigned)key; }

template <int KC>
__device__ __forceinline__ void list_insert(float x, int v, float (&val)[KC], int (&idx)[KC]) {
    // ids arrive in increasing order within a lane, so a strict comparison keeps the lower id first
    if (x > val[KC - 1]) {
        val[KC - 1] = x;
        idx[KC - 1] = v;
#pragma unroll
        for (int j = KC - 1; j > 0; --j) {
            if (val[j] > val[j - 1]) {
                float tv = val[j]; val[j] = val[j - 1]; val[j - 1] = tv;
                int ti = idx[j]; idx[j] = idx[j - 1]; idx[j - 1] = ti;
            }
        }
    }
}

template <bool BF16, int KC>
__global__ __launch_bounds__(LM_THREADS, 2)
void lmhead_kernel(const uint8_t* __restrict__ W, int row_bytes, int V,
                   const uint8_t* __restrict__ Hraw, int64_t h_seq_bytes, int M, int F, int B,
                   unsigned* __restrict__ done_count, float* __restrict__ part_ms, float* __restrict__ part_val, int* __restrict__ part_idx,
                   float* __restrict__ logits_out, int logit_rows_per_seq, int logit_row_base) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m16 = lane & 15, g = lane >> 4;          // MFMA lane coordinates
    const int r_in = lane >> 4, c16 = lane & 15;       // load coordinates: 4 rows x 256 B per instruction
    const int G = gridDim.x, mblk = blockIdx.y;
    const int wave_bytes = row_bytes >> 2;             // K bytes owned by this wave
    const int nst = wave_bytes / LM_CHUNK;
    const int ntask = (V + LM_ROWS - 1) / LM_ROWS;
    // workgroup bx owns a contiguous block of tasks (2 MB runs of W at the LLaMA shapes)
    const int tq = ntask / G, tr = ntask - tq * G;
    const int my_tasks = tq + ((int)blockIdx.x < tr ? 1 : 0);
    const int task_first = (int)blockIdx.x * tq + min((int)blockIdx.x, tr);
    const int total = my_tasks * nst;
    uint8_t* stage = smem + w * LM_STAGE;
    const int mrow = mblk * 16 + m16;                  // frontier row owned by this lane
    const bool row_valid = mrow < M;

    u32x4 R[LM_LOADS];
    auto issue = [&](int it) {
        const int task = task_first + it / nst;
        const int st = it - (it / nst) * nst;
        const size_t kb = (size_t)w * wave_bytes + (size_t)st * LM_CHUNK + c16 * 16;
#pragma unroll
        for (int j = 0; j < LM_LOADS; ++j) {
            int row = task * LM_ROWS + j * 4 + r_in;
            row = row < V ? row : V - 1;               // ragged tail: re-read the last row, masked later
            R[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(W + (size_t)row * row_bytes + kb));
        }
    };
    // The first stage of W is requested before anything else is set up: the row pointers of the optional
    // logits, the frontier-row divisions and the list initialisation below then run under that latency.
    if (total > 0) issue(0);
    __builtin_amdgcn_sched_barrier(0);

    if (blockIdx.x == 0 && mblk == 0)                   // counters of the merge kernel's last-arrival test
        for (int i = tid; i < B; i += LM_THREADS) done_count[i] = 0u;

    float run_m = -INFINITY, run_s = 0.f;
    float tval[KC];
    int tidx[KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) { tval[j] = -INFINITY; tidx[j] = INT_MAX; }

    // Raw logits (optional) are kept in registers for up to LOGIT_BUF finished tasks and leave
    // in one burst through an LDS transpose: wave w stores frontier rows w, w+4, w+8, w+12, each
    // quarter-wave 256 contiguous bytes.  Stores sprinkled into the read stream cost far more
    // than their bytes (the HBM channels keep turning around), so they are clustered in time.
    constexpr int LOGIT_BUF = 4;
    constexpr int LT_RS = LOGIT_BUF * LM_ROWS + 4;     // floats per row of the transpose tile (+16 B pad)
    float* lrow[4] = {nullptr, nullptr, nullptr, nullptr};
    if (logits_out != nullptr) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int wr = mblk * 16 + q * 4 + w;
            if (wr < M) {
                const int b = wr / F, s = wr - b * F;
                lrow[q] = logits_out + ((size_t)b * logit_rows_per_seq + logit_row_base + s) * (size_t)V;
            }
        }
    }
    floatx4 xs[LOGIT_BUF];
    int nbuf = 0, buf_task0 = task_first;
    auto flush_logits = [&]() {                        // called by the whole workgroup; stages must be idle
        float* lt = reinterpret_cast<float*>(smem);
#pragma unroll
        for (int t = 0; t < LOGIT_BUF; ++t)
            if (t < nbuf) *reinterpret_cast<floatx4*>(lt + m16 * LT_RS + t * LM_ROWS + w * 16 + g * 4) = xs[t];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // quarter-wave r_in takes buffered task r_in of row 4q + w: the wave writes one 1 KB run
            const int v0 = (buf_task0 + r_in) * LM_ROWS + c16 * 4;
            if (lrow[q] != nullptr && r_in < nbuf && v0 < V) {
                const floatx4 y = *reinterpret_cast<const floatx4*>(lt + (q * 4 + w) * LT_RS + r_in * LM_ROWS + c16 * 4);
                if (v0 + 3 < V && (V & 3) == 0) {
                    __builtin_nontemporal_store(y, reinterpret_cast<floatx4*>(lrow[q] + v0));
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) if (v0 + i < V) lrow[q][v0 + i] = y[i];
                }
            }
        }
        __syncthreads();                               // lt aliases the staging buffers
        buf_task0 += nbuf;
        nbuf = 0;
    };

    floatx4 acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // H fragments are fetched one stage ahead and *before* the next stage's W loads are issued:
    // loads retire in order, so a younger H load would otherwise make the MFMAs wait for the
    // whole W prefetch.
    auto frag0 = [&](int it) {
        const int st = it - (it / nst) * nst;
        return (w * wave_bytes + st * LM_CHUNK) >> 6;
    };
    // H fragments come straight from the caller's H: lane (m16, g) reads 16 bytes at
    // 64*frag + 16*g of frontier row m16 (rows beyond M are zero)
    const uint8_t* hrow = nullptr;
    if (row_valid) {
        const int b = mrow / F, s = mrow - b * F;
        hrow = Hraw + (int64_t)b * h_seq_bytes + (int64_t)s * row_bytes + g * 16;
    }
    auto load_h = [&](int fi) -> u32x4 {
        return hrow ? *reinterpret_cast<const u32x4*>(hrow + (size_t)fi * 64) : u32x4{0u, 0u, 0u, 0u};
    };
    u32x4 hf[LM_CHUNK / 64], hn[LM_CHUNK / 64];
    if (total > 0) {
#pragma unroll
        for (int t = 0; t < LM_CHUNK / 64; ++t) hn[t] = load_h(frag0(0) + t);
    }
    for (int it = 0; it < total; ++it) {
        const int ti = it / nst;
        const int st = it - ti * nst;
        const int task = task_first + ti;
#pragma unroll
        for (int j = 0; j < LM_LOADS; ++j)
            *reinterpret_cast<u32x4*>(stage + (j * 4 + r_in) * LM_RS + ((c16 ^ ((j * 4 + r_in) & 15)) << 4)) = R[j];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");    // stages are wave-private: no workgroup barrier
#pragma unroll
        for (int t = 0; t < LM_CHUNK / 64; ++t) hf[t] = hn[t];
        if (it + 1 < total) {
            const int f1 = frag0(it + 1);
#pragma unroll
            for (int t = 0; t < LM_CHUNK / 64; ++t) hn[t] = load_h(f1 + t);
            issue(it + 1);
        }

#pragma unroll
        for (int t = 0; t < LM_CHUNK / 64; ++t) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const u32x4 wf = *reinterpret_cast<const u32x4*>(
                    stage + (nb * 16 + m16) * LM_RS + (((t * 4 + g) ^ m16) << 4));
                if constexpr (BF16) {
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, wf), __builtin_bit_cast(bf16x8, hf[t]), acc[nb], 0, 0, 0);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                            __uint_as_float(wf[e]), __uint_as_float(hf[t][e]), acc[nb], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (st == nst - 1) __syncthreads();            // the reduction below reuses every wave's stage

        if (st == nst - 1) {
            // split-K reduction: wave w collects vocab-row block w from all four waves
            floatx4* red = reinterpret_cast<floatx4*>(smem);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                red[(w * 4 + nb) * 64 + lane] = acc[nb];
                acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
            __syncthreads();
            floatx4 x = red[(0 * 4 + w) * 64 + lane];
#pragma unroll
            for (int sw = 1; sw < 4; ++sw) x += red[(sw * 4 + w) * 64 + lane];
            __syncthreads();                           // red aliases the staging buffers

            const int vbase = task * LM_ROWS + w * 16 + g * 4;
            if (logits_out != nullptr) {               // uniform over the workgroup
#pragma unroll
                for (int t = 0; t < LOGIT_BUF; ++t) if (t == nbuf) xs[t] = x;
                ++nbuf;
                if (nbuf == LOGIT_BUF || ti == my_tasks - 1) flush_logits();
            }
            if (row_valid && vbase < V) {
                float xm = x[0];
#pragma unroll
                for (int i = 1; i < 4; ++i) if (vbase + i < V) xm = fmaxf(xm, x[i]);
                if (xm > run_m) { run_s *= __expf(run_m - xm); run_m = xm; }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (vbase + i < V) {
                        run_s += __expf(x[i] - run_m);
                        list_insert<KC>(x[i], vbase + i, tval, tidx);
                    }
                }
            }
        }
    }

    // ---- merge the 16 per-lane states of each frontier row (4 lane groups x 4 waves) in one 16-way
    // merge: every lane leaves its state in LDS, then the 16 lists of a row sit in the 16 lanes of one DPP
    // row (wave w takes frontier rows 4w .. 4w+3) and the best head is found with four row-local
    // butterfly steps per output element; the four waves work on different rows at the same time ----
    __syncthreads();                                                   // the staging buffers are idle
    // One LDS row of LM_MROW words per list position (and two more for max and sum-exp); the lane of wave a
    // sits at word 68 a + lane, so that both the writes (consecutive lanes) and the reads below (row r16 of
    // wave a, lane group b: word 68 a + 16 b + r16, with four consecutive r16 per wave) touch 64 different banks.
    constexpr int LM_MROW = 4 * 68;
    float* l_val = reinterpret_cast<float*>(smem);                     // [KC][LM_MROW]
    int* l_idx = reinterpret_cast<int*>(smem + KC * LM_MROW * 4);
    float* l_ms = reinterpret_cast<float*>(smem + 2 * KC * LM_MROW * 4);   // [2][LM_MROW]
    {
        const int me = w * 68 + lane;
#pragma unroll
        for (int j = 0; j < KC; ++j) { l_val[j * LM_MROW + me] = tval[j]; l_idx[j * LM_MROW + me] = tidx[j]; }
        l_ms[me] = run_m;
        l_ms[LM_MROW + me] = run_s;
    }
    __syncthreads();
    const int r16 = w * 4 + (lane >> 4), q = lane & 15;               // frontier row (within the block) and list of this lane
    {
        const int src = (q >> 2) * 68 + (q & 3) * 16 + r16;           // wave q / 4, lane group q % 4, row r16
#pragma unroll
        for (int j = 0; j < KC; ++j) { tval[j] = l_val[j * LM_MROW + src]; tidx[j] = l_idx[j * LM_MROW + src]; }
        run_m = l_ms[src];
        run_s = l_ms[LM_MROW + src];
    }
#define E2_ROW_STEP(CTRL)                                                                       \
    {                                                                                           \
        const float om = dpp_mov<CTRL>(run_m), os = dpp_mov<CTRL>(run_s);                       \
        const float nm = fmaxf(run_m, om);                                                      \
        const float a = run_m > -INFINITY ? run_s * __expf(run_m - nm) : 0.f;                   \
        const float c = om > -INFINITY ? os * __expf(om - nm) : 0.f;                            \
        run_m = nm;                                                                             \
        run_s = a + c;                                                                          \
    }
    E2_ROW_STEP(DPP_XOR1) E2_ROW_STEP(DPP_XOR2) E2_ROW_STEP(DPP_HALF_MIRROR) E2_ROW_STEP(DPP_MIRROR)
#undef E2_ROW_STEP
    // (value, id) pairs as 64-bit keys: a step of the butterfly is two lane moves, one comparison, two selects
    unsigned klo[KC], khi[KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) {
        const unsigned long long key = order_key(tval[j], tidx[j]);
        klo[j] = (unsigned)key;
        khi[j] = (unsigned)(key >> 32);
    }
    const unsigned long long empty = order_key(-INFINITY, INT_MAX);
    float mv[KC];
    int mi[KC];
#pragma unroll
    for (int rr = 0; rr < KC; ++rr) {
        unsigned blo = klo[0], bhi = khi[0];
#define E2_ROW_STEP(CTRL)                                                                       \
        {                                                                                       \
            const unsigned olo = (unsigned)dpp_mov<CTRL>((int)blo), ohi = (unsigned)dpp_mov<CTRL>((int)bhi); \
            const bool take = (((unsigned long long)ohi << 32) | olo) > (((unsigned long long)bhi << 32) | blo); \
            blo = take ? olo : blo;                                                             \
            bhi = take ? ohi : bhi;                                                             \
        }
        E2_ROW_STEP(DPP_XOR1) E2_ROW_STEP(DPP_XOR2) E2_ROW_STEP(DPP_HALF_MIRROR) E2_ROW_STEP(DPP_MIRROR)
#undef E2_ROW_STEP
        if (klo[0] == blo && khi[0] == bhi) {          // the list that held the winner moves up (ids are unique)
#pragma unroll
            for (int qq = 0; qq < KC - 1; ++qq) { klo[qq] = klo[qq + 1]; khi[qq] = khi[qq + 1]; }
            klo[KC - 1] = (unsigned)empty; khi[KC - 1] = (unsigned)(empty >> 32);
        }
        const unsigned long long best = ((unsigned long long)bhi << 32) | blo;
        mv[rr] = key_value(best); mi[rr] = key_id(best);
    }
    if (q == 0) {
        const size_t prow = (size_t)mblk * 16 + r16;                   // padded rows included
        part_ms[(prow * G + blockIdx.x) * 2 + 0] = run_m;
        part_ms[(prow * G + blockIdx.x) * 2 + 1] = run_s;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            part_val[(prow * G + blockIdx.x) * KC + j] = mv[j];
            part_idx[(prow * G + blockIdx.x) * KC + j] = mi[j];
        }
    }
}

// ---- many frontier rows (more than one 16-row block: batched serving) -----------------------
// With M > 16 rows the per-lane statistics of lmhead_kernel no longer fit in registers, and
// re-streaming W once per 16-row block multiplies the HBM traffic.  Instead W is streamed once
// for up to 160 rows: lmhead_gemm_kernel writes the raw logits [M, V] (to the caller's
// draft_logits rows, else to the workspace) and row_expand_kernel reads each row once for its
// (max, sum-exp, top-k), children and share of the frontier selection.
constexpr int GB_MBMAX = 10;                 // 16-row blocks per workgroup pass (160 frontier rows)
constexpr int GB_CHUNK = 256;                // bytes of K per row per stage
constexpr int GB_WSTAGE = LM_ROWS * GB_CHUNK;            // 16 KB of W per stage

// Destination of frontier row m's logits: the caller's [B, R, V] tensor or the dense workspace.
__device__ __forceinline__ float* logit_row_ptr(int m, int F, int V, float* logits_ws, float* logits_out,
                                                int logit_rows_per_seq, int logit_row_base) {
    if (logits_out == nullptr) return logits_ws + (size_t)m * V;
    const int b = m / F, s = m - b * F;
    return logits_out + ((size_t)b * logit_rows_per_seq + logit_row_base + s) * (size_t)V;
}

// Frontier rows re-tiled into MFMA B-fragment order (a fragment = 16 rows x 64 bytes of K = 64 lanes
// x 16 bytes, contiguous): Hp[block of 16 rows][64-byte K step][lane][16 B].  H is small (M x K), so
// this pre-pass costs a few microseconds; it lets the GEMM's waves fetch their fragments with
// fully coalesced 1 KiB loads straight into registers instead of staging H through LDS.
__global__ __launch_bounds__(256)
void pack_h_kernel(const uint8_t* __restrict__ Hraw, int64_t h_seq_bytes, int row_bytes, int M, int F,
                   u32x4* __restrict__ Hp, size_t npieces) {
    const int ksteps = row_bytes / 64;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < npieces; i += (size_t)gridDim.x * 256) {
        const int lane = (int)(i & 63), m16 = lane & 15, g = lane >> 4;
        const size_t frag = i >> 6;
        const int kstep = (int)(frag % ksteps);
        const int m = (int)(frag / ksteps) * 16 + m16;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (m < M) {
            const int b = m / F, s = m - b * F;
            v = *reinterpret_cast<const u32x4*>(Hraw + (int64_t)b * h_seq_bytes + (int64_t)s * row_bytes + (size_t)kstep * 64 + g * 16);
        }
        Hp[i] = v;
    }
}

// Workgroup = 4 waves, task = 64 vocab rows x the whole K; a stage is 256 bytes of K.  The W stage
// goes through LDS (XOR-swizzled 16-byte slots, two buffers, one barrier per stage) and is shared
// by the waves; the frontier fragments come from the re-tiled copy Hp (L2 hits), each fragment
// loaded by the one wave that needs it.  Wave (kh, mh) multiplies K half kh of the stage for half
// mh of the frontier blocks (at most five) with all four 16-row W blocks: the four waves carry
// the same number of MFMAs, and a W fragment feeds up to five of them.  At the end of a task the
// two K halves are added through LDS, each wave finishing two of the four W blocks.  In registers,
// W runs two stages ahead of the multiplication and the frontier fragments one.
constexpr int GB_RED = 4 * (GB_MBMAX / 2) * 2 * 64 * 16;   // bytes of the end-of-task exchange area
constexpr int GB_SMEM = 2 * GB_WSTAGE + GB_RED;

template <bool BF16>
__global__ __launch_bounds__(LM_THREADS, 2)
void lmhead_gemm_kernel(const uint8_t* __restrict__ W, int row_bytes, int V,
                        const uint8_t* __restrict__ Hp, int M, int F, int B,
                        unsigned* __restrict__ done_count, float* __restrict__ logits_ws,
                        float* __restrict__ logits_out, int logit_rows_per_seq, int logit_row_base) {
    constexpr int MH = GB_MBMAX / 2;                   // frontier blocks per wave
    constexpr int TH = GB_CHUNK / 128;                 // 64-byte K fragments per wave per stage
    extern __shared__ __align__(16) uint8_t smem[];
    floatx4* red = reinterpret_cast<floatx4*>(smem + 2 * GB_WSTAGE);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m16 = lane & 15, g = lane >> 4;          // MFMA lane coordinates
    const int r16 = tid >> 4, c16 = tid & 15;          // load coordinates: 16 rows x 256 B per instruction
    const int kh = w & 1, mh = w >> 1;
    const int G = gridDim.x;
    const int mb0 = blockIdx.y * GB_MBMAX;
    const int nmb = min(GB_MBMAX, (M + 15) / 16 - mb0);
    const int nlo = (nmb + 1) >> 1;
    const int mfirst = mh ? nlo : 0, mcnt = mh ? nmb - nlo : nlo;   // this wave's frontier blocks
    const int nst = row_bytes / GB_CHUNK;
    const int ksteps = row_bytes / 64;
    const int ntask = (V + LM_ROWS - 1) / LM_ROWS;
    const int tq = ntask / G, tr = ntask - tq * G;
    const int my_tasks = tq + ((int)blockIdx.x < tr ? 1 : 0);
    const int task_first = (int)blockIdx.x * tq + min((int)blockIdx.x, tr);
    const int total = my_tasks * nst;

    if (blockIdx.x == 0 && blockIdx.y == 0)            // counters of the merge kernel's last-arrival test
        for (int i = tid; i < B; i += LM_THREADS) done_count[i] = 0u;

    // this wave's fragments of stage 0 start here; block jj is ksteps KiB further, a stage 4 KiB
    const uint8_t* hbase = Hp + ((size_t)(mb0 + mfirst) * ksteps + kh * TH) * 1024 + lane * 16;
    float* lrow[MH];
#pragma unroll
    for (int jj = 0; jj < MH; ++jj) {
        const int m = (mb0 + mfirst + jj) * 16 + m16;
        lrow[jj] = (jj < mcnt && m < M) ? logit_row_ptr(m, F, V, logits_ws, logits_out, logit_rows_per_seq, logit_row_base)
                                        : nullptr;
    }

    // W is fetched two stages ahead (two register sets, used alternately), the frontier fragments
    // one stage ahead and *before* the younger W loads: loads retire in order, so the wait for a
    // stage's operands leaves the W loads of the stage after it in flight.
    u32x4 RWa[4], RWb[4], hn[MH][TH];
    auto issue_h = [&](int it) {
        const int st = it - (it / nst) * nst;
        const uint8_t* src = hbase + (size_t)st * (GB_CHUNK / 64) * 1024;
#pragma unroll
        for (int jj = 0; jj < MH; ++jj)
#pragma unroll
            for (int tt = 0; tt < TH; ++tt)
                if (jj < mcnt) hn[jj][tt] = *reinterpret_cast<const u32x4*>(src + ((size_t)jj * ksteps + tt) * 1024);
    };
    auto issue_w = [&](int it, u32x4 (&RW)[4]) {
        const int task = task_first + it / nst;
        const int st = it - (it / nst) * nst;
        const size_t kb = (size_t)st * GB_CHUNK;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int row = task * LM_ROWS + j * 16 + r16;
            row = row < V ? row : V - 1;               // ragged tail: re-read the last row, never stored
            RW[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(W + (size_t)row * row_bytes + kb + c16 * 16));
        }
    };

    floatx4 acc[MH][4];
#pragma unroll
    for (int jj = 0; jj < MH; ++jj)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[jj][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto step = [&](int it, u32x4 (&RW)[4], uint8_t* sW) {
        const int ti = it / nst;
        const int st = it - ti * nst;
        // this buffer was last read two stages ago, and every wave has passed a barrier since
#pragma unroll
        for (int j = 0; j < 4; ++j)
            *reinterpret_cast<u32x4*>(sW + (j * 16 + r16) * GB_CHUNK + ((c16 ^ r16) << 4)) = RW[j];
        u32x4 hf[MH][TH];
#pragma unroll
        for (int jj = 0; jj < MH; ++jj)
#pragma unroll
            for (int tt = 0; tt < TH; ++tt) hf[jj][tt] = hn[jj][tt];
        __syncthreads();
        if (it + 1 < total) issue_h(it + 1);
        if (it + 2 < total) issue_w(it + 2, RW);

#pragma unroll
        for (int tt = 0; tt < TH; ++tt) {
            const int t = kh * TH + tt;                // 64-byte K fragment of the stage
            u32x4 wf[4];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
                wf[nb] = *reinterpret_cast<const u32x4*>(sW + ((((nb + 2 * kh) & 3) * 16) + m16) * GB_CHUNK + (((t * 4 + g) ^ m16) << 4));
#pragma unroll
            for (int jj = 0; jj < MH; ++jj) {
                if (jj < mcnt) {                       // uniform over the wave
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        if constexpr (BF16) {
                            acc[jj][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, wf[nb]), __builtin_bit_cast(bf16x8, hf[jj][tt]), acc[jj][nb], 0, 0, 0);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                acc[jj][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                    __uint_as_float(wf[nb][e]), __uint_as_float(hf[jj][tt][e]), acc[jj][nb], 0, 0, 0);
                        }
                    }
                }
            }
        }

        if (st == nst - 1) {
            // Add the two K halves: wave kh finishes W blocks 2 kh and 2 kh + 1 (its accumulators 0, 1:
            // accumulator nb of wave kh belongs to W block (nb + 2 kh) mod 4, so that register
            // indices stay compile-time constants) and hands the other two to its partner through
            // LDS.  The area is written again only after the next task's barriers, which every
            // wave reaches after this read.
#pragma unroll
            for (int jj = 0; jj < MH; ++jj)
#pragma unroll
                for (int nl = 0; nl < 2; ++nl)
                    if (jj < mcnt) red[(((mh * 2 + (1 - kh)) * MH + jj) * 2 + nl) * 64 + lane] = acc[jj][2 + nl];
            __syncthreads();
            // output register i of W block nb: vocab row 64*task + 16*nb + 4*g + i, frontier row of lrow[jj]
            const int task = task_first + ti;
#pragma unroll
            for (int jj = 0; jj < MH; ++jj) {
#pragma unroll
                for (int nl = 0; nl < 2; ++nl) {
                    if (jj < mcnt) {
                        const floatx4 other = red[(((mh * 2 + kh) * MH + jj) * 2 + nl) * 64 + lane];
                        const floatx4 y = acc[jj][nl] + other;
                        const int v0 = task * LM_ROWS + (2 * kh + nl) * 16 + g * 4;
                        if (lrow[jj] != nullptr && v0 < V) {
                            if (v0 + 3 < V && (V & 3) == 0) {
                                *reinterpret_cast<floatx4*>(lrow[jj] + v0) = y;
                            } else {
#pragma unroll
                                for (int i = 0; i < 4; ++i) if (v0 + i < V) lrow[jj][v0 + i] = y[i];
                            }
                        }
                    }
                }
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) acc[jj][nb] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    if (total > 0) { issue_w(0, RWa); issue_h(0); }
    if (total > 1) issue_w(1, RWb);
    for (int it = 0; it < total; it += 2) {
        step(it, RWa, smem);
        if (it + 1 < total) step(it + 1, RWb, smem + GB_WSTAGE);
    }
}

// bf16, many rows: 128 vocab rows x up to 160 frontier rows per workgroup of 8 waves, one workgroup per
// compute unit, loading waves and multiplying waves.  Both operands are staged in LDS and shared; a step is
// 128 B of K of the W tile (128 rows) and of the frontier tile (160 rows), both rows x 128 B with swizzled
// 16-byte slots, both read from the caller's row-major tensors.  A compute unit therefore fetches every frontier
// row once per 128 vocab rows, where lmhead_gemm_kernel's four waves each fetch their own fragments per 64 rows.
// Waves 4-7 only load, straight from global memory into LDS (global_load_lds: no registers, no LDS
// writes by the waves): waves 4 and 5 stream 64 W rows each into a ring of five steps, four steps (64 KB per
// compute unit) ahead of the multiplication; waves 6 and 7 copy 80 frontier rows each from L2 into a
// ring of three, two steps ahead.  The two kinds of load sit in different waves because a wave's loads
// complete in order: waiting for a young frontier load would mean waiting for every older W load.  Waves 0-3
// only multiply: wave (wh, hh) takes vocab rows 64 wh .. +63 and frontier blocks 5 hh .. 5 hh + 4 over the
// whole K (no split-K), 20 MFMAs per 64-byte K step from 4 + 5 fragment reads out of the two tiles, and never issues a load, so a
// full memory pipeline stalls a loading wave, not the matrix cores.  One barrier per step.
constexpr int G2_THREADS = 512;
constexpr int G2_ROWS = 128;                           // vocab rows per task
constexpr int G2_WSTEP = G2_ROWS * 128;                // bytes of W per step (128 B of K per row)
constexpr int G2_HSTEP = GB_MBMAX * 16 * 128;          // bytes of the frontier tile per step (160 rows x 128 B of K)
constexpr int G2_WRING = 5, G2_HRING = 3;
constexpr int G2_SMEM = G2_WRING * G2_WSTEP + G2_HRING * G2_HSTEP;   // 143,360 of the 163,840 bytes

__global__ __launch_bounds__(G2_THREADS, 1)
void lmhead_gemm128_kernel(const uint8_t* __restrict__ W, int row_bytes, int V,
                           const uint8_t* __restrict__ Hraw, int64_t h_seq_bytes, int M, int F, int B,
                           unsigned* __restrict__ done_count, float* __restrict__ logits_ws,
                           float* __restrict__ logits_out, int logit_rows_per_seq, int logit_row_base) {
    typedef __attribute__((address_space(1))) const void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    constexpr int MH = GB_MBMAX / 2;                   // frontier blocks per multiplying wave
    __shared__ __align__(1024) uint8_t smem[G2_SMEM];
    uint8_t* const sW = smem;
    uint8_t* const sH = smem + G2_WRING * G2_WSTEP;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x;
    const int mb0 = blockIdx.y * GB_MBMAX;
    const int nmb = min(GB_MBMAX, (M + 15) / 16 - mb0);   // >= 1
    const int nstep = row_bytes / 128;                 // steps per task (>= 8)
    const int ntask = (V + G2_ROWS - 1) / G2_ROWS;
    const int tq = ntask / G, tr = ntask - tq * G;
    const int my_tasks = tq + ((int)blockIdx.x < tr ? 1 : 0);
    const int task_first = (int)blockIdx.x * tq + min((int)blockIdx.x, tr);
    const int total = my_tasks * nstep;

    if (blockIdx.x == 0 && blockIdx.y == 0)            // counters of the merge kernel's last-arrival test
        for (int i = tid; i < B; i += G2_THREADS) done_count[i] = 0u;

    if (w >= 6) {
        // ---- frontier waves: 80 of the 160 frontier rows each, straight from the caller's row-major rows (L2-resident:
        // 1.3 MB at 160 rows).  Like the W tile, a step of the frontier tile is rows x 128 B with swizzled 16-byte
        // slots; a load instruction fills 1 KiB = 8 rows x 128 B, lane (r, p) = (l / 8, l % 8).  Rows beyond M repeat
        // row M - 1 (their products are never stored). ----
        const int ph = w - 6;
        const int lr = lane >> 3, lp = lane & 7;
        const uint8_t* hsrc[10];                       // this lane's source row of each of the wave's ten instructions, at its piece
#pragma unroll
        for (int i = 0; i < 10; ++i) {
            const int rl = (ph * 10 + i) * 8 + lr;     // row inside the 160-row tile
            int m = mb0 * 16 + rl;
            m = m < M ? m : M - 1;
            const int b = m / F, sl = m - b * F;
            hsrc[i] = Hraw + (int64_t)b * h_seq_bytes + (int64_t)sl * row_bytes + ((lp ^ ((rl >> 1) & 7)) << 4);
        }
        int st = 0;                                    // step inside its task of the next step to request (no division per step)
        auto issue_h = [&](int h) {
            uint8_t* dst = sH + (h % G2_HRING) * G2_HSTEP;
#pragma unroll
            for (int i = 0; i < 10; ++i)
                __builtin_amdgcn_global_load_lds((gptr)(hsrc[i] + (size_t)st * 128), (lptr)(dst + (ph * 10 + i) * 1024), 16, 0, 0);
            st = st + 1 == nstep ? 0 : st + 1;
        };
        // a step's ten loads have landed once only those of younger steps are outstanding (in-order completion)
        auto wait_younger = [&](int n) {
            if (n >= 2) __builtin_amdgcn_s_waitcnt(0x4F74);        // vmcnt(20)
            else if (n == 1) __builtin_amdgcn_s_waitcnt(0x0F7A);   // vmcnt(10)
            else __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
        };
        static_assert(G2_HRING <= 3 && G2_WRING <= 7, "the waits cover two younger fragment steps and six younger W steps");
#pragma unroll
        for (int j = 0; j < G2_HRING; ++j) if (j < total) issue_h(j);
        if (total > 0) wait_younger(min(total - 1, G2_HRING - 1));
        __syncthreads();                               // step 0 is in LDS
        for (int h = 0; h < total; ++h) {
            if (h + 1 < total) wait_younger(min(total - 2 - h, G2_HRING - 2));
            __syncthreads();                           // step h is multiplied, step h + 1 is in LDS
            if (h + G2_HRING < total) issue_h(h + G2_HRING);
        }
    } else if (w >= 4) {
        // ---- W waves: 64 of the tile's 128 rows each; a load instruction fills 1 KiB of LDS = 8 rows x 128 B,
        // lane (r, p) = (l / 8, l % 8) owns position p of its row and fetches the source piece the swizzle puts
        // there.  Rows beyond V re-read the last row (never stored). ----
        const int pw = w - 4;
        int ti = 0, st = 0;                            // task and step inside it of the next step to request
        const int lr = lane >> 3, lp = lane & 7;
        auto issue_w = [&](int h) {
            const size_t kb = (size_t)st * 128;
            uint8_t* dst = sW + (h % G2_WRING) * G2_WSTEP;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int r0 = pw * 64 + i * 8, rl = r0 + lr;
                int row = (task_first + ti) * G2_ROWS + rl;
                row = row < V ? row : V - 1;
                const uint8_t* src = W + (size_t)row * row_bytes + kb + ((lp ^ ((rl >> 1) & 7)) << 4);
                __builtin_amdgcn_global_load_lds((gptr)src, (lptr)(dst + r0 * 128), 16, 0, 0);
            }
            if (++st == nstep) { st = 0; ++ti; }
        };
        auto wait_younger = [&](int n) {               // eight loads per step
            if (n >= 6) __builtin_amdgcn_s_waitcnt(0xCF70);        // vmcnt(48)
            else if (n == 5) __builtin_amdgcn_s_waitcnt(0x8F78);   // vmcnt(40)
            else if (n == 4) __builtin_amdgcn_s_waitcnt(0x8F70);   // vmcnt(32)
            else if (n == 3) __builtin_amdgcn_s_waitcnt(0x4F78);   // vmcnt(24)
            else if (n == 2) __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16)
            else if (n == 1) __builtin_amdgcn_s_waitcnt(0x0F78);   // vmcnt(8)
            else __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
        };
#pragma unroll
        for (int j = 0; j < G2_WRING; ++j) if (j < total) issue_w(j);
        if (total > 0) wait_younger(min(total - 1, G2_WRING - 1));
        __syncthreads();                               // step 0 is in LDS
        for (int h = 0; h < total; ++h) {
            if (h + 1 < total) wait_younger(min(total - 2 - h, G2_WRING - 2));
            __syncthreads();                           // step h is multiplied, step h + 1 is in LDS
            if (h + G2_WRING < total) issue_w(h + G2_WRING);
        }
    } else {
        // ---- multiplying waves ----
        const int m16 = lane & 15, g = lane >> 4;      // MFMA lane coordinates
        const int wh = w & 1, hh = w >> 1;
        const int hfirst = hh * MH;
        const int hcnt = max(0, min(MH, nmb - hfirst));   // this wave's frontier blocks (uniform)
        float* lrow[MH];
#pragma unroll
        for (int jj = 0; jj < MH; ++jj) {
            const int m = (mb0 + hfirst + jj) * 16 + m16;
            lrow[jj] = (jj < hcnt && m < M) ? logit_row_ptr(m, F, V, logits_ws, logits_out, logit_rows_per_seq, logit_row_base)
                                            : nullptr;
        }
        floatx4 acc[MH][4];
#pragma unroll
        for (int jj = 0; jj < MH; ++jj)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) acc[jj][nb] = floatx4{0.f, 0.f, 0.f, 0.f};
        // this lane's byte offset inside a W step for K step 0 of W block 0 (rows 16 nb + m16 share the swizzle)
        const unsigned wlane = (wh * 64 + m16) * 128;
        const int wswz = (m16 >> 1) & 7;
        __syncthreads();                               // step 0 is in LDS
        // FULL: the wave has all five frontier blocks -- straight-line code (all 18 fragment reads of a step are
        // requested up front; LDS returns them in order, so the first MFMAs start after five of them).  Otherwise
        // the blocks beyond hcnt are skipped with wave-uniform branches.
        auto run = [&](auto full_c) {
            constexpr bool FULL = decltype(full_c)::value;
            int ti = 0, st = 0;                        // task and step inside it (no division per step)
            for (int h = 0; h < total; ++h) {
                const uint8_t* wb = sW + (h % G2_WRING) * G2_WSTEP + wlane;
                const uint8_t* hb = sH + (h % G2_HRING) * G2_HSTEP + (hfirst * 16 + m16) * 128;
                u32x4 wf[2][4], hf[2][MH];
#pragma unroll
                for (int t = 0; t < 2; ++t) {          // 64-byte K steps of the step
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
                        wf[t][nb] = *reinterpret_cast<const u32x4*>(wb + nb * 16 * 128 + (((t * 4 + g) ^ wswz) << 4));
#pragma unroll
                    for (int jj = 0; jj < MH; ++jj)
                        if (FULL || jj < hcnt) hf[t][jj] = *reinterpret_cast<const u32x4*>(hb + jj * 16 * 128 + (((t * 4 + g) ^ wswz) << 4));
                }
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int jj = 0; jj < MH; ++jj)
                        if (FULL || jj < hcnt) {
#pragma unroll
                            for (int nb = 0; nb < 4; ++nb)
                                acc[jj][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    __builtin_bit_cast(bf16x8, wf[t][nb]), __builtin_bit_cast(bf16x8, hf[t][jj]), acc[jj][nb], 0, 0, 0);
                        }
                if (++st == nstep) {
                    // task finished: output register i of W block nb is vocab row 128 task + 64 wh + 16 nb + 4 g + i,
                    // frontier row of lrow[jj]
                    const int vb = (task_first + ti) * G2_ROWS + wh * 64 + g * 4;
#pragma unroll
                    for (int jj = 0; jj < MH; ++jj) {
#pragma unroll
                        for (int nb = 0; nb < 4; ++nb) {
                            const int v0 = vb + nb * 16;
                            if ((FULL || jj < hcnt) && lrow[jj] != nullptr && v0 < V) {
                                const floatx4 y = acc[jj][nb];
                                if (v0 + 3 < V && (V & 3) == 0) {
                                    *reinterpret_cast<floatx4*>(lrow[jj] + v0) = y;
                                } else {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) if (v0 + i < V) lrow[jj][v0 + i] = y[i];
                                }
                            }
                            acc[jj][nb] = floatx4{0.f, 0.f, 0.f, 0.f};
                        }
                    }
                    st = 0;
                    ++ti;
                }
                __syncthreads();                       // step h + 1 is in LDS; this step's buffers may be overwritten
            }
        };
        if (hcnt == MH) run(std::integral_constant<bool, true>{});
        else run(std::integral_constant<bool, false>{});
    }
}

// One workgroup per (frontier row, sequence).  Each of the G partial lists is sorted, so an
// entry can only be in the row's top k if its list's head is among the k best heads.  Heads,
// surviving entries (<= k*KC) and new candidates (frontier) are all ranked by counting.  The
// workgroup that finishes last for a sequence (a counter in the workspace, zeroed by
// lmhead_kernel) also selects the next frontier.
constexpr int MG_THREADS = 1024;
constexpr int MG_MAXN = EAGLE2_MAX_TOPK * EAGLE2_MAX_TOPK;   // most keys ranked at once

// Ranks of n <= MG_MAXN keys in LDS (descending; equal keys: lower position first), by all-pairs
// counting spread over the whole workgroup: with P threads per key (the largest power of two that
// fits MG_THREADS / n), thread
// (i, part) counts the keys j = part, part + P, ... that precede key i, and the partial counts meet
// in an LDS atomic.  rank[0..n) must be zero on entry; the caller synchronises before reading it.
__device__ __forceinline__ void rank_keys(const unsigned long long* keys, int n, int* rank, int tid) {
    const int lg = 31 - __clz(MG_THREADS / n);          // P = 2^lg threads per key: shifts instead of a division
    const int P = 1 << lg;
    const int i = tid >> lg, part = tid & (P - 1);
    if (i >= n) return;
    const unsigned long long ki = keys[i];
    int cnt = 0;
#pragma unroll 4
    for (int j = part; j < n; j += P) {
        const unsigned long long kj = keys[j];
        cnt += ((kj > ki) | ((kj == ki) & (j < i))) ? 1 : 0;   // (bitwise: no branches)
    }
    if (cnt) atomicAdd(rank + i, cnt);
}

// The end of a row's expansion, shared by both paths: ok[0..k) are the row's k best (value, token)
// keys, mx and log_sum its log-sum-exp; thread t < k holds the parent (par, ps) and writes child t.
// The workgroup that finishes last for a sequence (a counter in the workspace, zeroed by the
// LM-head kernel) also selects the next frontier.
__device__ __forceinline__ void finish_row(int d, int F, int k, int D, int C, int by_confidence, int static_tree,
                                           int par, double ps, float mx, const double* log_sum_lds,
                                           const unsigned long long* ok,
                                           int* __restrict__ cand_token, double* __restrict__ cand_score,
                                           int* __restrict__ cand_parent, int* __restrict__ frontier,
                                           unsigned* __restrict__ done_count) {
    __shared__ unsigned long long s_fk[MG_MAXN];        // new candidates' scores (frontier selection)
    __shared__ int s_frank[MG_MAXN];
    __shared__ int s_last;
    const int slot = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int base = d == 0 ? 0 : k + (d - 1) * k * k;
    if (tid < MG_MAXN) s_frank[tid] = 0;
    if (tid < k) {
        const double log_sum = *log_sum_lds;
        const int cid = base + slot * k + tid;
        const unsigned long long key = ok[tid];
        const float ov = key != 0ull ? key_value(key) : -INFINITY;
        const double sc = ps + (((double)ov - (double)mx) - log_sum);
        cand_token[(size_t)b * C + cid] = key != 0ull ? key_id(key) : 0;
        cand_parent[(size_t)b * C + cid] = par;
        // The score is also read by the workgroup that picks the next frontier, possibly on
        // another XCD: store it at device scope (write-through to the coherence point) instead of
        // a device-scope fence (which writes back the whole L2).  These stores and the counter
        // increment below are all issued by wave 0; the wave waits here until every one of its
        // outstanding stores has been acknowledged, so the counter cannot overtake a score.
        __hip_atomic_store(cand_score + (size_t)b * C + cid, sc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        wait_vector_memory();
    }
    if (d + 1 >= D || static_tree) return;               // a static shape fixes the frontiers beforehand

    // the last workgroup of this sequence picks the next frontier
    __syncthreads();
    if (tid == 0) {
        const unsigned prev = __hip_atomic_fetch_add(done_count + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = prev == (unsigned)(F - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last) return;
    const int nn = F * k;                               // <= MG_MAXN new candidates, in candidate-id order
    if (tid < nn) {
        double key = __hip_atomic_load(cand_score + (size_t)b * C + base + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (by_confidence && d > 0) {                   // "w/o value" (Section 5.2): the node's own log confidence
            int par = frontier[((size_t)b * D + d) * k + tid / k];
            if (par < 0 || par >= C) par = 0;
            key -= cand_score[(size_t)b * C + par];     // written by an earlier pass
        }
        s_fk[tid] = order_key(key);
    }
    __syncthreads();
    rank_keys(s_fk, nn, s_frank, tid);
    __syncthreads();
    if (tid < nn) {
        const int r = s_frank[tid];
        if (r < k) frontier[((size_t)b * D + d + 1) * k + r] = base + tid;
    }
}


// The merge of one (frontier row, sequence): ms, pv and pi are that row's G partial pairs and lists,
// in global memory or in LDS.
template <int KC>
__device__ __forceinline__ void merge_row(int d, int F, int k, int D, int C, int G, int by_confidence, int static_tree,
                                          const float* __restrict__ ms, const float* __restrict__ pv,
                                          const int* __restrict__ pi,
                                          int* __restrict__ cand_token, double* __restrict__ cand_score,
                                          int* __restrict__ cand_parent, int* __restrict__ frontier,
                                          unsigned* __restrict__ done_count) {
    constexpr int NW = MG_THREADS / 64;
    __shared__ float s_f[NW];
    __shared__ double s_d[NW];
    __shared__ unsigned long long s_wk[NW * EAGLE2_MAX_TOPK];   // per-wave winners among the list heads: key, list
    __shared__ int s_wl[NW * EAGLE2_MAX_TOPK];
    __shared__ unsigned long long s_ck[MG_MAXN];        // entries of the surviving lists
    __shared__ unsigned long long s_ok[EAGLE2_MAX_TOPK];   // the row's k best
    __shared__ int s_rank[2][MG_MAXN];                  // one set of counters per ranking, zeroed once
    __shared__ double s_logsum;
    static_assert(NW * EAGLE2_MAX_TOPK <= MG_MAXN, "the per-wave winners are ranked like the other key sets");
    const int slot = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    // loads first: the parent and its score (two dependent global loads, needed only at the end),
    // the heads of the G lists and the (max, sum-exp) pairs
    int par = -1;
    double ps = 0.0;
    if (d > 0 && tid < k) {
        par = frontier[((size_t)b * D + d) * k + slot];
        if (par < 0 || par >= C) par = 0;               // garbage in the caller's frontier stays in bounds
        ps = cand_score[(size_t)b * C + par];
    }
    float my_m = -INFINITY, my_s = 0.f;
    unsigned long long hk = 0ull;                       // this thread's list head (0 ranks after every real key)
    if (tid < G) {
        hk = order_key(pv[(size_t)tid * KC], pi[(size_t)tid * KC]);
        my_m = ms[tid * 2];
        my_s = ms[tid * 2 + 1];
    }
    if (tid < EAGLE2_MAX_TOPK) s_ok[tid] = 0ull;
    if (tid < MG_MAXN) { s_rank[0][tid] = 0; s_rank[1][tid] = 0; s_wk[tid] = 0ull; s_ck[tid] = 0ull; s_wl[tid] = 0; }
    // log-sum-exp over the G partial pairs
    float mloc = wave_max(my_m);
    if (lane == 0) s_f[wave] = mloc;
    __syncthreads();
    float mx = s_f[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, s_f[w]);
    double sloc = my_m > -INFINITY ? (double)my_s * exp((double)my_m - (double)mx) : 0.0;
    sloc = wave_sum(sloc);
    if (lane == 0) s_d[wave] = sloc;

    // the k best heads: inside every wave each head counts the heads of the other lanes that precede
    // it (broadcast with v_readlane, no LDS); the at most k survivors per wave are then ranked
    // against each other
    const int nlive = G < k ? G : k;
    const int nwv = (G + 63) >> 6;                          // waves that hold heads
    if (wave < nwv) {
        const int klo = (int)(unsigned)hk, khi = (int)(unsigned)(hk >> 32);
        int r = 0;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            const unsigned long long kj = ((unsigned long long)(unsigned)read_lane(khi, j) << 32) | (unsigned)read_lane(klo, j);
            r += kj > hk ? 1 : 0;                       // equal keys are empty lists only, which never contribute
        }
        if (r < nlive && tid < G) { s_wk[wave * nlive + r] = hk; s_wl[wave * nlive + r] = tid; }
    }
    __syncthreads();
    const int n2 = nwv * nlive;                             // <= MG_MAXN survivors, compact in s_wk
    rank_keys(s_wk, n2, s_rank[0], tid);
    __syncthreads();
    // a winner of rank r < nlive brings in its list: nlive * KC candidates in all
    const int ncand = nlive * KC;
    if (tid == MG_THREADS - 1) {                        // an idle thread takes the logarithm while the lists are fetched
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += s_d[w];
        s_logsum = log(tot);
    }
    if (tid < n2) {
        const int r = s_rank[0][tid], l = s_wl[tid];
        if (r < nlive && s_wk[tid] != 0ull && l >= 0 && l < G) {
#pragma unroll
            for (int j = 0; j < KC; ++j) s_ck[r * KC + j] = order_key(pv[(size_t)l * KC + j], pi[(size_t)l * KC + j]);
        }
    }
    __syncthreads();
    rank_keys(s_ck, ncand, s_rank[1], tid);
    __syncthreads();
    if (tid < ncand) {
        const int r = s_rank[1][tid];
        const unsigned long long key = s_ck[tid];
        if (r < k && key != 0ull && key_id(key) != INT_MAX) s_ok[r] = key;
    }
    __syncthreads();
    finish_row(d, F, k, D, C, by_confidence, static_tree, par, ps, mx, &s_logsum, s_ok, cand_token, cand_score, cand_parent,
               frontier, done_count);
}

template <int KC>
__global__ __launch_bounds__(MG_THREADS)
void expand_merge_kernel(int d, int F, int k, int D, int C, int G, int by_confidence, int static_tree,
                         const float* __restrict__ part_ms, const float* __restrict__ part_val,
                         const int* __restrict__ part_idx,
                         int* __restrict__ cand_token, double* __restrict__ cand_score,
                         int* __restrict__ cand_parent, int* __restrict__ frontier,
                         unsigned* __restrict__ done_count) {
    const size_t prow = (size_t)blockIdx.y * F + blockIdx.x;
    merge_row<KC>(d, F, k, D, C, G, by_confidence, static_tree, part_ms + prow * G * 2, part_val + prow * G * KC,
                  part_idx + prow * G * KC, cand_token, cand_score, cand_parent, frontier, done_count);
}

// The many-row path's second half: one workgroup per (frontier row, sequence) reads the row's V raw
// logits once, 16 per thread and iteration, and does everything else.  Log-sum-exp: every wave
// keeps a running maximum and its lanes their share of the sum of exponentials.  Top k: the k-th
// largest of all wave maxima seen so far (each wave's values are disjoint) is a lower bound of the
// row's k-th largest value, so only the few values at or above it are candidates; they are appended
// to a list in LDS (most waves have none and skip the step) and ranked by counting at the end.
// A row with so many equal values that the list overflows is redone by k exact selection sweeps.
constexpr int RX_STEP = MG_THREADS * 16;     // vocabulary entries per workgroup iteration
constexpr int RX_CAP = MG_MAXN;              // candidates ranked at once

__device__ __forceinline__ void load_row_piece(const float* __restrict__ src, int c0, int V, bool vec, int tid, float (&x)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = c0 + (i * MG_THREADS + tid) * 4;
        if (vec && v + 3 < V) {
            const floatx4 y = *reinterpret_cast<const floatx4*>(src + v);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[i * 4 + e] = y[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[i * 4 + e] = v + e < V ? src[v + e] : -INFINITY;
        }
    }
}

template <int KC>
__global__ __launch_bounds__(MG_THREADS)
void row_expand_kernel(int V, int d, int F, int k, int D, int C, int by_confidence, int static_tree,
                       const float* __restrict__ logits_ws, const float* __restrict__ logits_out,
                       int logit_rows_per_seq, int logit_row_base,
                       int* __restrict__ cand_token, double* __restrict__ cand_score,
                       int* __restrict__ cand_parent, int* __restrict__ frontier,
                       unsigned* __restrict__ done_count) {
    constexpr int NW = MG_THREADS / 64;
    static_assert(NW + KC <= 64 && KC <= NW, "wave maxima and the running best are ranked by one wave; the first iteration must yield k maxima");
    __shared__ float s_wm[2][NW];                       // this iteration's wave maxima
    __shared__ float s_best[2][EAGLE2_MAX_TOPK];        // the KC largest wave maxima so far
    __shared__ float s_m[NW], s_s[NW];
    __shared__ unsigned long long s_ck[RX_CAP];
    __shared__ int s_rank[RX_CAP];
    __shared__ unsigned long long s_ok[EAGLE2_MAX_TOPK];
    __shared__ unsigned long long s_pick;
    __shared__ int s_n;
    __shared__ double s_logsum;
    const int slot = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = b * F + slot;
    const float* src = logit_row_ptr(m, F, V, const_cast<float*>(logits_ws), const_cast<float*>(logits_out),
                                     logit_rows_per_seq, logit_row_base);
    const bool vec = (V & 3) == 0;
    float x[16], xn[16];
    load_row_piece(src, 0, V, vec, tid, x);
    // the parent and its score: two dependent global loads, needed only at the end
    int par = -1;
    double ps = 0.0;
    if (d > 0 && tid < k) {
        par = frontier[((size_t)b * D + d) * k + slot];
        if (par < 0 || par >= C) par = 0;               // garbage in the caller's frontier stays in bounds
        ps = cand_score[(size_t)b * C + par];
    }
    if (tid == 0) s_n = 0;
    if (tid < EAGLE2_MAX_TOPK) { s_ok[tid] = 0ull; s_best[0][tid] = -INFINITY; s_best[1][tid] = -INFINITY; }
    if (tid < RX_CAP) { s_ck[tid] = 0ull; s_rank[tid] = 0; }
    float run_m = -INFINITY, run_s = 0.f;               // the wave's running maximum; this lane's share of the sum
    int it = 0;
    for (int c0 = 0; c0 < V; c0 += RX_STEP, it ^= 1) {
        if (c0 + RX_STEP < V) load_row_piece(src, c0 + RX_STEP, V, vec, tid, xn);   // in flight during this piece's work
        float mx = x[0];
#pragma unroll
        for (int q = 1; q < 16; ++q) mx = fmaxf(mx, x[q]);
        const float wm = wave_max(mx);
        if (lane == 0) s_wm[it][w] = wm;
        if (wm > -INFINITY) {                           // uniform over the wave: it holds at least one entry
            const float nm = fmaxf(run_m, wm);
            float sum = run_s * __expf(run_m - nm);     // 0 * exp(-inf) = 0 the first time
#pragma unroll
            for (int q = 0; q < 16; ++q) sum += __expf(x[q] - nm);   // exp(-inf) = 0 for the padding
            run_s = sum;
            run_m = nm;
        }
        __syncthreads();
        // Every wave ranks the NW new maxima and the KC best so far (one per lane, ties by lane) and
        // writes the new KC best: the same values from every wave.  The buffers alternate, and the
        // barrier above separates an iteration's reads from the next one's writes.
        const bool have = lane < NW + KC;
        const float cm = lane < NW ? s_wm[it][lane] : (have ? s_best[it ^ 1][lane - NW] : -INFINITY);
        int r = 0;
#pragma unroll
        for (int j = 0; j < NW + KC; ++j) {
            const float o = read_lane(cm, j);
            r += ((o > cm) | ((o == cm) & (j < lane))) ? 1 : 0;
        }
        if (have && r < KC) s_best[it][r] = cm;
        const float thr = wave_max(have && r == k - 1 ? cm : -INFINITY);
        if (__ballot(mx >= thr) != 0ull) {              // uniform over the wave; rare after the first iterations
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int v = c0 + ((q >> 2) * MG_THREADS + tid) * 4 + (q & 3);
                if (x[q] >= thr && v < V) {             // (the padding is -inf and passes a bound of -inf)
                    const int pos = atomicAdd(&s_n, 1);
                    if (pos < RX_CAP) s_ck[pos] = order_key(x[q], v);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) x[q] = xn[q];
    }
    run_s = wave_sumf(run_s);
    if (lane == 0) { s_m[w] = run_m; s_s[w] = run_s; }
    __syncthreads();
    float rmx = s_m[0];
#pragma unroll
    for (int j = 1; j < NW; ++j) rmx = fmaxf(rmx, s_m[j]);
    if (tid == MG_THREADS - 1) {                        // an otherwise idle thread takes the logarithm
        double tot = 0.0;
#pragma unroll
        for (int j = 0; j < NW; ++j) tot += s_m[j] > -INFINITY ? (double)s_s[j] * exp((double)s_m[j] - (double)rmx) : 0.0;
        s_logsum = log(tot);
    }
    const int n = s_n;
    if (n <= RX_CAP) {                                  // uniform over the workgroup
        if (n > 0) rank_keys(s_ck, n, s_rank, tid);
        __syncthreads();
        if (tid < n) {
            const int r = s_rank[tid];
            if (r < k) s_ok[r] = s_ck[tid];
        }
    } else {
        // k sweeps over the row, each taking the best key below the previous winner (keys are
        // unique: they carry the token id); slow and exact
        unsigned long long prev = ~0ull;
        for (int r = 0; r < k; ++r) {
            if (tid == 0) s_pick = 0ull;
            __syncthreads();
            unsigned long long best = 0ull;
            for (int v = tid; v < V; v += MG_THREADS) {
                const unsigned long long key = order_key(src[v], v);
                if (key < prev && key > best) best = key;
            }
            if (best != 0ull) atomicMax(&s_pick, best);
            __syncthreads();
            prev = s_pick;                              // 0 once the row is exhausted
            if (tid == 0) s_ok[r] = prev;
            __syncthreads();
        }
    }
    __syncthreads();
    finish_row(d, F, k, D, C, by_confidence, static_tree, par, ps, rmx, &s_logsum, s_ok, cand_token, cand_score, cand_parent,
               frontier, done_count);
}

// out[M, N] (float32, dense) = X[M, K] . W[N, K]^T for M > 16 rows: pack_h_kernel + lmhead_gemm_kernel.
// X row m = (b, s) lives at X + b * x_seq_bytes + s * row_bytes; hp_ws needs ceil(M/16)*16 * row_bytes bytes.
static int gemm128_grid(int n_rows) {                  // one workgroup per compute unit, at most one per task
    const int ntask = (n_rows + G2_ROWS - 1) / G2_ROWS;
    const int cus = device_cu_count();
    return ntask < cus ? ntask : cus;
}

int gemm_rows(bool bf16, const void* X, int64_t x_seq_bytes, int M, int F, const void* W, int N, int row_bytes,
              float* out, void* hp_ws, unsigned* done_count, int n_done, hipStream_t st) {
    const int mblks = (M + 15) / 16;
    const int ny = (mblks + GB_MBMAX - 1) / GB_MBMAX;
    if (bf16) {                                        // reads X as it lies
        hipLaunchKernelGGL(lmhead_gemm128_kernel, dim3(gemm128_grid(N), ny), dim3(G2_THREADS), 0, st, static_cast<const uint8_t*>(W),
                           row_bytes, N, static_cast<const uint8_t*>(X), x_seq_bytes, M, F, n_done, done_count, out,
                           static_cast<float*>(nullptr), 0, 0);
        E2_HIP(hipGetLastError());
        return EAGLE2_OK;
    }
    const int ntask = (N + LM_ROWS - 1) / LM_ROWS;
    int gg = 2 * device_cu_count();
    if (gg > ntask) gg = ntask;
    const size_t npieces = (size_t)mblks * 16 * row_bytes / 16;
    hipLaunchKernelGGL(pack_h_kernel, dim3((unsigned)((npieces + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint8_t*>(X), x_seq_bytes, row_bytes, M, F, static_cast<u32x4*>(hp_ws), npieces);
    E2_HIP(hipGetLastError());
    hipLaunchKernelGGL((lmhead_gemm_kernel<false>), dim3(gg, ny), dim3(LM_THREADS), GB_SMEM, st, static_cast<const uint8_t*>(W),
                       row_bytes, N, static_cast<const uint8_t*>(hp_ws), M, F, n_done, done_count, out,
                       static_cast<float*>(nullptr), 0, 0);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

static int lm_grid(const eagle2_cfg* cfg) {
    const int ntask = (cfg->vocab + LM_ROWS - 1) / LM_ROWS;
    int g = 2 * device_cu_count();                     // two resident workgroups per compute unit
    if (g > LM_GMAX) g = LM_GMAX;
    if (g > ntask) g = ntask;
    return g < 1 ? 1 : g;
}

struct ExpandWs { size_t ms, val, idx, cnt, logits, hp, total; };
static ExpandWs expand_layout(const eagle2_cfg* cfg) {
    const size_t mmax = (size_t)cfg->batch * cfg->topk;
    const size_t mblks = (mmax + 15) / 16;
    ExpandWs w;
    w.ms = 0;
    w.val = w.ms + round_up(mblks * 16 * LM_GMAX * 2 * sizeof(float), 256);
    w.idx = w.val + round_up(mblks * 16 * LM_GMAX * EAGLE2_MAX_TOPK * sizeof(float), 256);
    w.cnt = w.idx + round_up(mblks * 16 * LM_GMAX * EAGLE2_MAX_TOPK * sizeof(int), 256);
    w.logits = w.cnt + round_up((size_t)cfg->batch * sizeof(unsigned), 256);
    // dense [M, V] logits of the many-row path (used when the caller keeps no draft logits)
    w.hp = w.logits + (mmax > 16 ? round_up(mmax * (size_t)cfg->vocab * sizeof(float), 256) : 0);
    // frontier rows re-tiled into fragment order for the many-row path
    w.total = w.hp + (mmax > 16 ? round_up(mblks * 16 * (size_t)cfg->hidden * elem_size(cfg), 256) : 0);
    return w;
}
size_t expand_workspace(const eagle2_cfg* cfg) { return expand_layout(cfg).total; }

template <bool BF16, int KC>
static int launch_expand(const eagle2_cfg* cfg, int d, const void* H, int64_t h_seq_stride, const void* W,
                         int32_t* cand_token, double* cand_score, int32_t* cand_parent, int32_t* frontier,
                         float* draft_logits, uint8_t* ws, hipStream_t st) {
    const int k = cfg->topk, F = d == 0 ? 1 : k, M = cfg->batch * F;
    const int row_bytes = cfg->hidden * elem_size(cfg);
    const int mblks = (M + 15) / 16;
    const ExpandWs L = expand_layout(cfg);
    float* part_ms = reinterpret_cast<float*>(ws + L.ms);
    float* part_val = reinterpret_cast<float*>(ws + L.val);
    int* part_idx = reinterpret_cast<int*>(ws + L.idx);
    unsigned* done_count = reinterpret_cast<unsigned*>(ws + L.cnt);
    const int64_t stride_el = h_seq_stride == 0 ? (int64_t)F * cfg->hidden : h_seq_stride;

    const int R = n_draft_rows(cfg);
    const int row_base = d == 0 ? 0 : 1 + (d - 1) * k;
    if (M > 16) {
        // many rows: stream W once per 160 rows into raw logits, then per-row statistics
        const int ntask = (cfg->vocab + LM_ROWS - 1) / LM_ROWS;
        int gg = 2 * device_cu_count();
        if (gg > ntask) gg = ntask;
        const int ny = (mblks + GB_MBMAX - 1) / GB_MBMAX;
        float* logits_ws = reinterpret_cast<float*>(ws + L.logits);
        if constexpr (BF16) {                          // reads H as it lies
            timing_begin(0, st);
            hipLaunchKernelGGL(lmhead_gemm128_kernel, dim3(gemm128_grid(cfg->vocab), ny), dim3(G2_THREADS), 0, st,
                               reinterpret_cast<const uint8_t*>(W), row_bytes, cfg->vocab, reinterpret_cast<const uint8_t*>(H),
                               stride_el * elem_size(cfg), M, F, cfg->batch, done_count, logits_ws, draft_logits, R, row_base);
        } else {
            uint8_t* Hp = ws + L.hp;
            const size_t npieces = (size_t)mblks * 16 * row_bytes / 16;
            hipLaunchKernelGGL(pack_h_kernel, dim3((unsigned)((npieces + 255) / 256)), dim3(256), 0, st,
                               reinterpret_cast<const uint8_t*>(H), stride_el * elem_size(cfg), row_bytes, M, F,
                               reinterpret_cast<u32x4*>(Hp), npieces);
            E2_HIP(hipGetLastError());
            timing_begin(0, st);
            hipLaunchKernelGGL((lmhead_gemm_kernel<BF16>), dim3(gg, ny), dim3(LM_THREADS), GB_SMEM, st,
                               reinterpret_cast<const uint8_t*>(W), row_bytes, cfg->vocab, Hp, M, F, cfg->batch, done_count,
                               logits_ws, draft_logits, R, row_base);
        }
        timing_end(0, st);
        E2_HIP(hipGetLastError());
        hipLaunchKernelGGL((row_expand_kernel<KC>), dim3(F, cfg->batch), dim3(MG_THREADS), 0, st, cfg->vocab,
                           d, F, k, cfg->depth, n_cand(cfg), (cfg->flags & EAGLE2_FLAG_RANK_BY_CONFIDENCE) ? 1 : 0,
                           (cfg->flags & EAGLE2_FLAG_STATIC_TREE) ? 1 : 0, logits_ws, draft_logits, R, row_base,
                           cand_token, cand_score, cand_parent, frontier, done_count);
        E2_HIP(hipGetLastError());
        return EAGLE2_OK;
    }
    const int G = lm_grid(cfg);
    {
        const size_t smem = 4 * LM_STAGE;
        static_assert(4 * LM_STAGE >= (2 * EAGLE2_MAX_TOPK + 2) * 4 * 68 * 4, "merge area must fit");
        timing_begin(0, st);
        hipLaunchKernelGGL((lmhead_kernel<BF16, KC>), dim3(G, mblks), dim3(LM_THREADS), smem, st,
                           reinterpret_cast<const uint8_t*>(W), row_bytes, cfg->vocab,
                           reinterpret_cast<const uint8_t*>(H), stride_el * elem_size(cfg), M, F, cfg->batch, done_count,
                           part_ms, part_val, part_idx, draft_logits, R, row_base);
        timing_end(0, st);
        E2_HIP(hipGetLastError());
    }

    hipLaunchKernelGGL((expand_merge_kernel<KC>), dim3(F, cfg->batch), dim3(MG_THREADS), 0, st,
                       d, F, k, cfg->depth, n_cand(cfg), G, (cfg->flags & EAGLE2_FLAG_RANK_BY_CONFIDENCE) ? 1 : 0,
                       (cfg->flags & EAGLE2_FLAG_STATIC_TREE) ? 1 : 0, part_ms, part_val, part_idx,
                       cand_token, cand_score, cand_parent, frontier, done_count);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_expand(const eagle2_cfg* cfg, int32_t d, const void* H, int64_t h_seq_stride, const void* W,
                             int32_t* cand_token, double* cand_score, int32_t* cand_parent,
                             int32_t* frontier, float* draft_logits,
                             void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(d >= 0 && d < cfg->depth, EAGLE2_ERR_ARG, "eagle2_expand: pass index %d outside [0, %d)", d, cfg->depth);
    E2_REQUIRE(H && W && cand_token && cand_score && cand_parent && frontier, EAGLE2_ERR_ARG,
               "eagle2_expand: null pointer argument");
    E2_REQUIRE(aligned16(H) && aligned16(W) && aligned16(draft_logits), EAGLE2_ERR_ARG,
               "eagle2_expand: H, W and draft_logits must be 16-byte aligned");
    const int F = d == 0 ? 1 : cfg->topk;
    E2_REQUIRE(h_seq_stride == 0 || h_seq_stride >= (int64_t)F * cfg->hidden, EAGLE2_ERR_ARG,
               "eagle2_expand: h_seq_stride %lld smaller than one sequence's rows", (long long)h_seq_stride);
    E2_REQUIRE((h_seq_stride * elem_size(cfg)) % 16 == 0, EAGLE2_ERR_ARG, "eagle2_expand: h_seq_stride not 16-byte aligned");
    E2_REQUIRE(workspace && workspace_bytes >= expand_workspace(cfg), EAGLE2_ERR_WORKSPACE,
               "eagle2_expand: workspace of %zu bytes, need %zu", workspace_bytes, expand_workspace(cfg));
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = cfg->dtype == EAGLE2_DTYPE_BF16;
    const int k = cfg->topk;
#define E2_GO(BF, KC) return launch_expand<BF, KC>(cfg, d, H, h_seq_stride, W, cand_token, cand_score, cand_parent, frontier, draft_logits, ws, st)
    if (bf) { if (k <= 4) E2_GO(true, 4); else if (k <= 10) E2_GO(true, 10); else E2_GO(true, 16); }
    else    { if (k <= 4) E2_GO(false, 4); else if (k <= 10) E2_GO(false, 10); else E2_GO(false, 16); }
#undef E2_GO
}
