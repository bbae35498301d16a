// Expansion phase (Section 4.1 of the EAGLE-2 paper): draft LM-head projection of the
// frontier rows, log-softmax, per-row top-k, joint-score accumulation along the path
// (value equation of Section 4.1, as a sum of logs) and selection of the next frontier.
//
// Three kernels per pass:
//   pack_h_kernel       frontier hidden states -> MFMA operand order (tiny)
//   lmhead_kernel       streams W once from HBM; per workgroup and frontier row it
//                       emits a partial (max, sum-exp, top-k) over the vocab rows it saw
//   expand_merge_kernel merges the partials, appends the k children per row with their
//                       joint scores and picks the next frontier
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

namespace eagle2 {

constexpr int LM_THREADS = 256;
constexpr int LM_ROWS = 64;                  // vocab rows per task
constexpr int LM_CHUNK = 256;                // bytes per row per stage per wave
constexpr int LM_RS = LM_CHUNK;              // LDS row stride; 16-byte slots are XOR-swizzled by the row
constexpr int LM_STAGE = LM_ROWS * LM_RS;    // bytes of LDS per wave (4 waves: 64 KB)
constexpr int LM_LOADS = LM_ROWS * LM_CHUNK / 1024;   // 16-byte loads per lane per stage
constexpr int LM_GMAX = 1024;                // upper bound on workgroups (partials per row)

__global__ void pack_h_kernel(const uint8_t* __restrict__ H, int64_t seq_stride_bytes, int row_bytes,
                              int M, int F, u32x4* __restrict__ Hp, unsigned* __restrict__ done_count, int B) {
    const int nfrag = row_bytes / 64;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.y == 0)                                // counters of the merge kernel's last-arrival test
        for (int i = gid; i < B; i += gridDim.x * blockDim.x) done_count[i] = 0u;
    const int fi = gid >> 6, lane = gid & 63;
    if (fi >= nfrag) return;
    const int mblk = blockIdx.y;
    const int f = lane & 15, g = lane >> 4;
    const int m = mblk * 16 + f;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (m < M) {
        const int b = m / F, s = m - b * F;
        const uint8_t* src = H + (int64_t)b * seq_stride_bytes + (int64_t)s * row_bytes + fi * 64 + g * 16;
        v = *reinterpret_cast<const u32x4*>(src);
    }
    Hp[((size_t)mblk * nfrag + fi) * 64 + lane] = v;
}

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
                   const u32x4* __restrict__ Hp, int M, int F,
                   float* __restrict__ part_ms, float* __restrict__ part_val, int* __restrict__ part_idx,
                   float* __restrict__ logits_out, int logit_rows_per_seq, int logit_row_base) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m16 = lane & 15, g = lane >> 4;          // MFMA lane coordinates
    const int r_in = lane >> 4, c16 = lane & 15;       // load coordinates: 4 rows x 256 B per instruction
    const int G = gridDim.x, mblk = blockIdx.y;
    const int nfrag = row_bytes >> 6;
    const int wave_bytes = row_bytes >> 2;             // K bytes owned by this wave
    const int nst = wave_bytes / LM_CHUNK;
    const int ntask = (V + LM_ROWS - 1) / LM_ROWS;
    const int my_tasks = ((int)blockIdx.x < ntask) ? (ntask - (int)blockIdx.x + G - 1) / G : 0;
    const int total = my_tasks * nst;
    uint8_t* stage = smem + w * LM_STAGE;
    const int mrow = mblk * 16 + m16;                  // frontier row owned by this lane
    const bool row_valid = mrow < M;

    float run_m = -INFINITY, run_s = 0.f;
    float tval[KC];
    int tidx[KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) { tval[j] = -INFINITY; tidx[j] = INT_MAX; }

    float* lrow = nullptr;
    if (logits_out != nullptr && row_valid) {
        const int b = mrow / F, s = mrow - b * F;
        lrow = logits_out + ((size_t)b * logit_rows_per_seq + logit_row_base + s) * (size_t)V;
    }

    u32x4 R[LM_LOADS];
    auto issue = [&](int it) {
        const int task = blockIdx.x + (it / nst) * G;
        const int st = it - (it / nst) * nst;
        const size_t kb = (size_t)w * wave_bytes + (size_t)st * LM_CHUNK + c16 * 16;
#pragma unroll
        for (int j = 0; j < LM_LOADS; ++j) {
            int row = task * LM_ROWS + j * 4 + r_in;
            row = row < V ? row : V - 1;               // ragged tail: re-read the last row, masked later
            R[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(W + (size_t)row * row_bytes + kb));
        }
    };

    floatx4 acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (total > 0) issue(0);
    for (int it = 0; it < total; ++it) {
        const int ti = it / nst;
        const int st = it - ti * nst;
        const int task = blockIdx.x + ti * G;
#pragma unroll
        for (int j = 0; j < LM_LOADS; ++j)
            *reinterpret_cast<u32x4*>(stage + (j * 4 + r_in) * LM_RS + ((c16 ^ ((j * 4 + r_in) & 15)) << 4)) = R[j];
        __syncthreads();
        if (it + 1 < total) issue(it + 1);

        const int fi0 = (w * wave_bytes + st * LM_CHUNK) >> 6;
        u32x4 hf[LM_CHUNK / 64];
#pragma unroll
        for (int t = 0; t < LM_CHUNK / 64; ++t)
            hf[t] = Hp[((size_t)mblk * nfrag + fi0 + t) * 64 + lane];
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
        __syncthreads();                               // all waves are done reading their stage

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
            if (row_valid && vbase < V) {
                if (lrow != nullptr) {
                    if (vbase + 3 < V && (V & 3) == 0) {
                        *reinterpret_cast<floatx4*>(lrow + vbase) = x;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) if (vbase + i < V) lrow[vbase + i] = x[i];
                    }
                }
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

    // ---- merge the 16 per-lane states of each frontier row (4 lane groups x 4 waves) ----
    __syncthreads();
    float* l_val = reinterpret_cast<float*>(smem);                 // [16 rows][16 src][KC]
    int* l_idx = reinterpret_cast<int*>(smem + 16 * 16 * KC * 4);
    float* l_ms = reinterpret_cast<float*>(smem + 2 * 16 * 16 * KC * 4);   // [16][16][2]
    {
        const int src = w * 4 + g;
        const int base = (m16 * 16 + src) * KC;
#pragma unroll
        for (int j = 0; j < KC; ++j) { l_val[base + j] = tval[j]; l_idx[base + j] = tidx[j]; }
        l_ms[(m16 * 16 + src) * 2 + 0] = run_m;
        l_ms[(m16 * 16 + src) * 2 + 1] = run_s;
    }
    __syncthreads();
    if (tid < 16) {
        const int f = tid;
        const int prow = mblk * 16 + f;                // partial row index (padded rows included)
        float mx = -INFINITY;
        for (int s = 0; s < 16; ++s) mx = fmaxf(mx, l_ms[(f * 16 + s) * 2]);
        float sm = 0.f;
        for (int s = 0; s < 16; ++s) {
            const float ms = l_ms[(f * 16 + s) * 2];
            if (ms > -INFINITY) sm += l_ms[(f * 16 + s) * 2 + 1] * __expf(ms - mx);
        }
        part_ms[((size_t)prow * G + blockIdx.x) * 2 + 0] = mx;
        part_ms[((size_t)prow * G + blockIdx.x) * 2 + 1] = sm;
        // 16-way merge of sorted lists: heads in registers, one LDS read per output
        float hv[16]; int hi[16]; int hp[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) { hv[s] = l_val[(f * 16 + s) * KC]; hi[s] = l_idx[(f * 16 + s) * KC]; hp[s] = 0; }
        for (int j = 0; j < KC; ++j) {
            int bs = 0; float bv = hv[0]; int bi = hi[0];
#pragma unroll
            for (int s = 1; s < 16; ++s)
                if (ranks_before(hv[s], hi[s], bv, bi)) { bv = hv[s]; bi = hi[s]; bs = s; }
            part_val[((size_t)prow * G + blockIdx.x) * KC + j] = bv;
            part_idx[((size_t)prow * G + blockIdx.x) * KC + j] = bi;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                if (s == bs) {
                    const int np = hp[s] + 1;
                    hp[s] = np;
                    if (np < KC) { hv[s] = l_val[(f * 16 + s) * KC + np]; hi[s] = l_idx[(f * 16 + s) * KC + np]; }
                    else { hv[s] = -INFINITY; hi[s] = INT_MAX; }
                }
            }
        }
    }
}

// butterfly arg-best over a wave: every lane ends with the best (value, index)
__device__ __forceinline__ void wave_best(float& v, int& i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(i, o, 64);
        if (ranks_before(ov, oi, v, i)) { v = ov; i = oi; }
    }
}
__device__ __forceinline__ void wave_best(double& v, int& i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(i, o, 64);
        if (ranks_before(ov, oi, v, i)) { v = ov; i = oi; }
    }
}

// One workgroup per (frontier row, sequence).  Threads stride over the row's G*KC partial
// candidates keeping a sorted top-KC each; waves, then the workgroup, reduce those lists by
// repeated arg-best.  The workgroup that finishes last for a sequence (a counter in the
// workspace, zeroed by pack_h_kernel) also selects the next frontier.
constexpr int MG_THREADS = 256;

template <int KC>
__device__ __forceinline__ void full_insert(float x, int v, float (&val)[KC], int (&idx)[KC]) {
    if (ranks_before(x, v, val[KC - 1], idx[KC - 1])) {
        val[KC - 1] = x; idx[KC - 1] = v;
#pragma unroll
        for (int q = KC - 1; q > 0; --q) {
            if (ranks_before(val[q], idx[q], val[q - 1], idx[q - 1])) {
                float tv = val[q]; val[q] = val[q - 1]; val[q - 1] = tv;
                int ti = idx[q]; idx[q] = idx[q - 1]; idx[q - 1] = ti;
            }
        }
    }
}

// k rounds of wave-wide arg-best over the lanes' sorted lists; lane r ends up holding the
// r-th best (value, index) of the wave in (out_v, out_i)
template <int KC>
__device__ __forceinline__ void wave_topk(float (&val)[KC], int (&idx)[KC], int k, int lane, float& out_v, int& out_i) {
    out_v = -INFINITY; out_i = INT_MAX;
    for (int r = 0; r < k; ++r) {
        float bv = val[0]; int bi = idx[0];
        wave_best(bv, bi);
        if (val[0] == bv && idx[0] == bi) {            // the winner pops its head
#pragma unroll
            for (int q = 0; q < KC - 1; ++q) { val[q] = val[q + 1]; idx[q] = idx[q + 1]; }
            val[KC - 1] = -INFINITY; idx[KC - 1] = INT_MAX;
        }
        if (lane == r) { out_v = bv; out_i = bi; }
    }
}

template <int KC>
__global__ __launch_bounds__(MG_THREADS)
void expand_merge_kernel(int d, int F, int k, int D, int C, int G,
                         const float* __restrict__ part_ms, const float* __restrict__ part_val,
                         const int* __restrict__ part_idx,
                         int* __restrict__ cand_token, double* __restrict__ cand_score,
                         int* __restrict__ cand_parent, int* __restrict__ frontier,
                         unsigned* __restrict__ done_count) {
    constexpr int NW = MG_THREADS / 64;
    __shared__ float s_f[NW];
    __shared__ double s_d[NW];
    __shared__ float s_cv[NW * EAGLE2_MAX_TOPK];
    __shared__ int s_ci[NW * EAGLE2_MAX_TOPK];
    __shared__ int s_last;
    const int slot = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int base = d == 0 ? 0 : k + (d - 1) * k * k;
    const size_t prow = (size_t)b * F + slot;

    // log-sum-exp over the G partial (max, sum) pairs
    const float* ms = part_ms + prow * G * 2;
    float mloc = -INFINITY;
    for (int p = tid; p < G; p += MG_THREADS) mloc = fmaxf(mloc, ms[p * 2]);
    mloc = wave_max(mloc);
    if (lane == 0) s_f[wave] = mloc;
    __syncthreads();
    float mx = s_f[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, s_f[w]);
    double sloc = 0.0;
    for (int p = tid; p < G; p += MG_THREADS) {
        const float mp = ms[p * 2];
        if (mp > -INFINITY) sloc += (double)ms[p * 2 + 1] * exp((double)mp - (double)mx);
    }
    sloc = wave_sum(sloc);
    if (lane == 0) s_d[wave] = sloc;

    // per-thread top-KC over its share of the candidates (loads batched four at a time)
    float tval[KC]; int tidx[KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) { tval[j] = -INFINITY; tidx[j] = INT_MAX; }
    const float* pv = part_val + prow * G * KC;
    const int* pi = part_idx + prow * G * KC;
    const int n = G * KC;
    for (int j0 = tid; j0 < n; j0 += 4 * MG_THREADS) {
        float xv[4]; int xi[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * MG_THREADS;
            xv[u] = j < n ? pv[j] : -INFINITY;
            xi[u] = j < n ? pi[j] : INT_MAX;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) full_insert<KC>(xv[u], xi[u], tval, tidx);
    }
    float wv; int wi;
    wave_topk<KC>(tval, tidx, k, lane, wv, wi);
    if (lane < k) { s_cv[wave * k + lane] = wv; s_ci[wave * k + lane] = wi; }
    __syncthreads();
    double log_sum = 0.0;
    if (wave == 0) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += s_d[w];
        log_sum = log(tot);
        // NW*k <= 64 candidates, one per lane
        float cv[1] = {lane < NW * k ? s_cv[lane] : -INFINITY};
        int ci[1] = {lane < NW * k ? s_ci[lane] : INT_MAX};
        float my_x; int my_tok;
        wave_topk<1>(cv, ci, k, lane, my_x, my_tok);
        if (lane < k) {
            const int cid = base + slot * k + lane;
            int par = d == 0 ? -1 : frontier[((size_t)b * D + d) * k + slot];
            if (d > 0 && (par < 0 || par >= C)) par = 0;   // garbage in the caller's frontier stays in bounds
            const double ps = d == 0 ? 0.0 : cand_score[(size_t)b * C + par];
            cand_token[(size_t)b * C + cid] = my_tok;
            cand_score[(size_t)b * C + cid] = ps + (((double)my_x - (double)mx) - log_sum);
            cand_parent[(size_t)b * C + cid] = par;
        }
    }
    if (d + 1 >= D) return;

    // the last workgroup of this sequence picks the next frontier
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        const unsigned prev = atomicAdd(done_count + b, 1u);
        s_last = prev == (unsigned)(F - 1) ? 1 : 0;
        __threadfence();
    }
    __syncthreads();
    if (!s_last || wave != 0) return;
    const int nn = F * k;                               // <= 256 new candidates, <= 4 per lane
    double v[4]; int id[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int j = lane + q * 64;
        v[q] = j < nn ? __hip_atomic_load(cand_score + (size_t)b * C + base + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                      : -INFINITY;
        id[q] = j < nn ? base + j : INT_MAX;
    }
    int mine = -1;
    for (int r = 0; r < k; ++r) {
        double bv = v[0]; int bi = id[0];
#pragma unroll
        for (int q = 1; q < 4; ++q) if (ranks_before(v[q], id[q], bv, bi)) { bv = v[q]; bi = id[q]; }
        wave_best(bv, bi);
#pragma unroll
        for (int q = 0; q < 4; ++q) if (id[q] == bi) { v[q] = -INFINITY; id[q] = INT_MAX; }
        if (lane == r) mine = bi;
    }
    if (lane < k) frontier[((size_t)b * D + d + 1) * k + lane] = mine;
}

static int lm_grid(const eagle2_cfg* cfg) {
    const int ntask = (cfg->vocab + LM_ROWS - 1) / LM_ROWS;
    int g = 2 * device_cu_count();
    if (g > LM_GMAX) g = LM_GMAX;
    if (g > ntask) g = ntask;
    return g < 1 ? 1 : g;
}

struct ExpandWs { size_t hp, ms, val, idx, cnt, total; };
static ExpandWs expand_layout(const eagle2_cfg* cfg) {
    const size_t row_bytes = (size_t)cfg->hidden * elem_size(cfg);
    const size_t mmax = (size_t)cfg->batch * cfg->topk;
    const size_t mblks = (mmax + 15) / 16;
    ExpandWs w;
    w.hp = 0;
    w.ms = round_up(mblks * row_bytes * 16, 256);
    w.val = w.ms + round_up(mblks * 16 * LM_GMAX * 2 * sizeof(float), 256);
    w.idx = w.val + round_up(mblks * 16 * LM_GMAX * EAGLE2_MAX_TOPK * sizeof(float), 256);
    w.cnt = w.idx + round_up(mblks * 16 * LM_GMAX * EAGLE2_MAX_TOPK * sizeof(int), 256);
    w.total = w.cnt + round_up((size_t)cfg->batch * sizeof(unsigned), 256);
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
    const int G = lm_grid(cfg);
    const ExpandWs L = expand_layout(cfg);
    u32x4* Hp = reinterpret_cast<u32x4*>(ws + L.hp);
    float* part_ms = reinterpret_cast<float*>(ws + L.ms);
    float* part_val = reinterpret_cast<float*>(ws + L.val);
    int* part_idx = reinterpret_cast<int*>(ws + L.idx);
    unsigned* done_count = reinterpret_cast<unsigned*>(ws + L.cnt);
    const int64_t stride_el = h_seq_stride == 0 ? (int64_t)F * cfg->hidden : h_seq_stride;

    const int nfrag = row_bytes / 64;
    dim3 pg((nfrag * 64 + 255) / 256, mblks);
    hipLaunchKernelGGL(pack_h_kernel, pg, dim3(256), 0, st, reinterpret_cast<const uint8_t*>(H),
                       stride_el * elem_size(cfg), row_bytes, M, F, Hp, done_count, cfg->batch);
    E2_HIP(hipGetLastError());

    const size_t smem = 4 * LM_STAGE;
    static_assert(4 * LM_STAGE >= 2 * 16 * 16 * EAGLE2_MAX_TOPK * 4 + 16 * 16 * 2 * 4, "merge area must fit");
    const int R = n_draft_rows(cfg);
    const int row_base = d == 0 ? 0 : 1 + (d - 1) * k;
    timing_begin(0, st);
    hipLaunchKernelGGL((lmhead_kernel<BF16, KC>), dim3(G, mblks), dim3(LM_THREADS), smem, st,
                       reinterpret_cast<const uint8_t*>(W), row_bytes, cfg->vocab, Hp, M, F,
                       part_ms, part_val, part_idx, draft_logits, R, row_base);
    timing_end(0, st);
    E2_HIP(hipGetLastError());

    hipLaunchKernelGGL((expand_merge_kernel<KC>), dim3(F, cfg->batch), dim3(MG_THREADS), 0, st,
                       d, F, k, cfg->depth, n_cand(cfg), G, part_ms, part_val, part_idx,
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
