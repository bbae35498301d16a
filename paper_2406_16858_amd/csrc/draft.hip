// Forward pass of the draft model between two expansion passes (Section 2.2 of the EAGLE-2
// paper, "Drafting Stage": autoregression at the feature level, with the token sequence advanced
// by one step; Section 4.1: all nodes of the current layer go through the draft model in one
// pass under tree attention).  The paper does not print the draft network; this is one
// LLaMA-style decoder layer (RMSNorm, rotary grouped-query attention, SwiGLU MLP, residuals)
// behind a linear fusion of [token embedding ; previous feature].
//
// The five weight matrices are streamed once per pass by linear_kernel, the LM-head streaming
// kernel without its statistics: 64 output rows per task, split-K over the four waves of a
// workgroup, and -- because these matrices have far fewer rows than a vocabulary -- split-K
// over workgroups too (grid z), each slice writing its own float32 partial.  The small
// kernels between them add the slices up and apply the element-wise steps; the SwiGLU step runs
// in the task ends of the gate / up product where that product is not split over workgroups.

#include "common.h"

namespace eagle2 {

constexpr int DL_THREADS = 256;
constexpr int DL_ROWS = 64;                  // output rows per task
constexpr int DL_CHUNK = 256;                // bytes of K per row per stage per wave
constexpr int DL_STAGE = DL_ROWS * DL_CHUNK;
constexpr int DL_LOADS = DL_ROWS * DL_CHUNK / 1024;

__device__ __forceinline__ float to_float(const void* p, size_t i, bool bf16) {
    if (!bf16) return static_cast<const float*>(p)[i];
    return __uint_as_float((unsigned)static_cast<const uint16_t*>(p)[i] << 16);
}
__device__ __forceinline__ void from_float(void* p, size_t i, float v, bool bf16) {
    if (!bf16) { static_cast<float*>(p)[i] = v; return; }
    const __bf16 h = (__bf16)v;                        // round to nearest even
    static_cast<uint16_t*>(p)[i] = __builtin_bit_cast(uint16_t, h);
}
// part[slice][m_pad][N] = X[M, K-slice] . W[N, K-slice]^T.  Input row m = (b, s) lives at
// X + b * x_seq_bytes + s * row_bytes (the same addressing as the LM-head kernel's H).
//
// GLU: W is the gate matrix stacked on the up matrix ([2 * N, K]); a task is 32 gate rows and the
// 32 up rows of the same outputs, K is not split over workgroups, and the task's end writes
// act[m][n] = silu(gate) * up in the activation type instead of a float32 partial (N a multiple
// of 32): the element-wise kernel between the two MLP products and its launch fall away.
template <bool BF16, bool GLU>
__global__ __launch_bounds__(DL_THREADS, 2)
void linear_kernel(const uint8_t* __restrict__ W, int row_bytes, int N,
                   const uint8_t* __restrict__ Xraw, int64_t x_seq_bytes, int M, int F,
                   float* __restrict__ part, int m_pad, void* __restrict__ act) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m16 = lane & 15, g = lane >> 4;          // MFMA lane coordinates
    const int r_in = lane >> 4, c16 = lane & 15;       // load coordinates: 4 rows x 256 B per instruction
    const int G = gridDim.x, mblk = blockIdx.y, slice = blockIdx.z;
    // The row's 256-byte stages are dealt as evenly as possible to the 4 * slices (slice, wave) units,
    // consecutive stages per unit: K need only be a multiple of 256 bytes (units differ by one stage at most).
    const int stages = row_bytes / DL_CHUNK, units = 4 * (int)gridDim.z, unit = slice * 4 + w;
    const int sq = stages / units, sr = stages - sq * units;
    const int nst = sq + (unit < sr ? 1 : 0);          // >= 1: the host keeps 4 * slices <= stages
    const size_t kbase = (size_t)(unit * sq + min(unit, sr)) * DL_CHUNK;
    const int ntask = GLU ? N / 32 : (N + DL_ROWS - 1) / DL_ROWS;
    const int tq = ntask / G, tr = ntask - tq * G;
    const int my_tasks = tq + ((int)blockIdx.x < tr ? 1 : 0);
    const int task_first = (int)blockIdx.x * tq + min((int)blockIdx.x, tr);
    const int total = my_tasks * nst;
    uint8_t* stage = smem + w * DL_STAGE;
    const int mrow = mblk * 16 + m16;                  // input row owned by this lane

    u32x4 R[DL_LOADS];
    auto issue = [&](int it) {
        const int task = task_first + it / nst;
        const int st = it - (it / nst) * nst;
        const size_t kb = kbase + (size_t)st * DL_CHUNK + c16 * 16;
#pragma unroll
        for (int j = 0; j < DL_LOADS; ++j) {
            int row;
            if constexpr (GLU) {                       // local rows 0..31: gate, 32..63: up (matrix rows N + ...)
                row = task * 32 + (j * 4 + r_in) + (j >= DL_LOADS / 2 ? N - 32 : 0);
            } else {
                row = task * DL_ROWS + j * 4 + r_in;
                row = row < N ? row : N - 1;           // ragged tail: re-read the last row, never stored
            }
            R[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(W + (size_t)row * row_bytes + kb));
        }
    };
    floatx4 acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // input fragments: lane (m16, g) reads 16 bytes at 64*frag + 16*g of input row m16, one stage
    // ahead and before the next stage's W loads (loads retire in order)
    const uint8_t* xrow = nullptr;
    if (mrow < M) {
        const int b = mrow / F, s = mrow - b * F;
        xrow = Xraw + (int64_t)b * x_seq_bytes + (int64_t)s * row_bytes + kbase + g * 16;
    }
    auto load_x = [&](int st, int t) -> u32x4 {
        return xrow ? *reinterpret_cast<const u32x4*>(xrow + (size_t)st * DL_CHUNK + t * 64) : u32x4{0u, 0u, 0u, 0u};
    };
    u32x4 xf[DL_CHUNK / 64], xn[DL_CHUNK / 64];
    if (total > 0) {
#pragma unroll
        for (int t = 0; t < DL_CHUNK / 64; ++t) xn[t] = load_x(0, t);
        issue(0);
    }
    for (int it = 0; it < total; ++it) {
        const int ti = it / nst;
        const int st = it - ti * nst;
#pragma unroll
        for (int j = 0; j < DL_LOADS; ++j)
            *reinterpret_cast<u32x4*>(stage + (j * 4 + r_in) * DL_CHUNK + ((c16 ^ ((j * 4 + r_in) & 15)) << 4)) = R[j];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");    // stages are wave-private: no workgroup barrier
#pragma unroll
        for (int t = 0; t < DL_CHUNK / 64; ++t) xf[t] = xn[t];
        if (it + 1 < total) {
            const int st1 = (it + 1) - ((it + 1) / nst) * nst;
#pragma unroll
            for (int t = 0; t < DL_CHUNK / 64; ++t) xn[t] = load_x(st1, t);
            issue(it + 1);
        }
#pragma unroll
        for (int t = 0; t < DL_CHUNK / 64; ++t) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const u32x4 wf = *reinterpret_cast<const u32x4*>(
                    stage + (nb * 16 + m16) * DL_CHUNK + (((t * 4 + g) ^ m16) << 4));
                if constexpr (BF16) {
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, wf), __builtin_bit_cast(bf16x8, xf[t]), acc[nb], 0, 0, 0);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                            __uint_as_float(wf[e]), __uint_as_float(xf[t][e]), acc[nb], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (st == nst - 1) {
            // split-K reduction over the four waves: wave w collects output-row block w
            __syncthreads();
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
            if constexpr (GLU) {
                // waves 0 and 1 hold gate rows 16w + 4g + i; the up rows of the same outputs are blocks w + 2
                floatx4 up = red[(0 * 4 + (w | 2)) * 64 + lane];
#pragma unroll
                for (int sw = 1; sw < 4; ++sw) up += red[(sw * 4 + (w | 2)) * 64 + lane];
                __syncthreads();                       // red aliases the staging buffers
                const int n0 = (task_first + ti) * 32 + w * 16 + g * 4;
                if (w < 2 && mrow < M) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        from_float(act, (size_t)mrow * N + n0 + i, x[i] / (1.f + __expf(-x[i])) * up[i], BF16);
                }
                continue;
            }
            __syncthreads();                           // red aliases the staging buffers
            // register i: output row 64*task + 16*w + 4*g + i of input row mrow
            const int n0 = (task_first + ti) * DL_ROWS + w * 16 + g * 4;
            if (mrow < M && n0 < N) {
                float* dst = part + ((size_t)slice * m_pad + mrow) * N + n0;
                if (n0 + 3 < N && (N & 3) == 0) {
                    *reinterpret_cast<floatx4*>(dst) = x;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) if (n0 + i < N) dst[i] = x[i];
                }
            }
        }
    }
}

// ---- element-wise kernels: one workgroup per input row m = (b, s) -------------------------------

__device__ __forceinline__ float sum_slices(const float* part, int S, int m_pad, int m, int N, int n) {
    const float* p = part + (size_t)m * N + n;
    const size_t step = (size_t)m_pad * N;
    float v = 0.f;
    int s = 0;
    for (; s + 4 <= S; s += 4)                         // independent loads
        v += (p[(size_t)s * step] + p[(size_t)(s + 1) * step]) + (p[(size_t)(s + 2) * step] + p[(size_t)(s + 3) * step]);
    for (; s < S; ++s) v += p[(size_t)s * step];
    return v;
}
// four consecutive outputs n .. n+3 (n a multiple of 4, N a multiple of 4): the slices' loads are independent
__device__ __forceinline__ floatx4 sum_slices4(const float* part, int S, int m_pad, int m, int N, int n) {
    floatx4 v = {0.f, 0.f, 0.f, 0.f};
    const float* p = part + (size_t)m * N + n;
    const size_t step = (size_t)m_pad * N;
    int s = 0;
    for (; s + 4 <= S; s += 4) {
        const floatx4 a = *reinterpret_cast<const floatx4*>(p + (size_t)s * step);
        const floatx4 b = *reinterpret_cast<const floatx4*>(p + (size_t)(s + 1) * step);
        const floatx4 c = *reinterpret_cast<const floatx4*>(p + (size_t)(s + 2) * step);
        const floatx4 d = *reinterpret_cast<const floatx4*>(p + (size_t)(s + 3) * step);
        v += (a + b) + (c + d);
    }
    for (; s < S; ++s) v += *reinterpret_cast<const floatx4*>(p + (size_t)s * step);
    return v;
}
// draft row of frontier slot s of pass d, and of its parent
__device__ __forceinline__ int draft_row_of(int d, int s, int k) { return d == 0 ? 0 : 1 + (d - 1) * k + s; }

// x_in[m] = [embed[token] ; feature of the parent position]; mask and position of the row.
__global__ __launch_bounds__(DL_THREADS)
void draft_gather_kernel(int d, int F, int k, int D, int C, int Hd, int Rd, int words, int V, bool bf16,
                         const int* __restrict__ cand_token, const int* __restrict__ cand_parent,
                         const int* __restrict__ frontier, const int* __restrict__ root_token,
                         const void* __restrict__ root_feature, const int* __restrict__ prefix_len,
                         const void* __restrict__ embed, const void* __restrict__ draft_feature,
                         unsigned long long* __restrict__ draft_mask, void* __restrict__ x_in, int* __restrict__ pos) {
    const int m = blockIdx.x, b = m / F, s = m - b * F, tid = threadIdx.x;
    const int row = draft_row_of(d, s, k);
    int token, prow = -1;                              // parent's draft row, -1: the position before the root
    if (d == 0) {
        token = root_token[b];
    } else {
        int c = frontier[((size_t)b * D + d) * k + s];
        if (c < 0 || c >= C) c = 0;                    // garbage in the caller's arrays stays in bounds
        token = cand_token[(size_t)b * C + c];
        const int p = cand_parent[(size_t)b * C + c];
        prow = 0;                                      // children of the root
        if (d >= 2) {
            for (int sp = 0; sp < k; ++sp)
                if (frontier[((size_t)b * D + d - 1) * k + sp] == p) prow = draft_row_of(d - 1, sp, k);
        }
    }
    if (token < 0 || token >= V) token = 0;
    // both halves are plain row copies in the activation type: 16-byte pieces (rows are multiples of 1 KiB)
    const int es = bf16 ? 2 : 4, nvec = Hd * es / 16;
    const u32x4* e_src = reinterpret_cast<const u32x4*>(static_cast<const uint8_t*>(embed) + (size_t)token * Hd * es);
    const u32x4* f_src = prow < 0
        ? reinterpret_cast<const u32x4*>(static_cast<const uint8_t*>(root_feature) + (size_t)b * Hd * es)
        : reinterpret_cast<const u32x4*>(static_cast<const uint8_t*>(draft_feature) + ((size_t)b * Rd + prow) * Hd * es);
    u32x4* dst = reinterpret_cast<u32x4*>(static_cast<uint8_t*>(x_in) + (size_t)m * 2 * Hd * es);
    for (int i = tid; i < nvec; i += DL_THREADS) {
        dst[i] = e_src[i];
        dst[nvec + i] = f_src[i];
    }
    if (tid < words) {
        unsigned long long bits = prow < 0 ? 0ull : draft_mask[((size_t)b * Rd + prow) * words + tid];
        if ((row >> 6) == tid) bits |= 1ull << (row & 63);
        draft_mask[((size_t)b * Rd + row) * words + tid] = bits;
    }
    if (tid == 0) pos[m] = prefix_len[b] + d;
}

// x = sum of the slices (+ residual); n = rmsnorm(x) * gain in the activation type.  One workgroup
// of 1024 threads per row, four consecutive elements per thread and step (Hd is a multiple of 256).
constexpr int RN_THREADS = 1024;
__global__ __launch_bounds__(RN_THREADS)
void sum_rmsnorm_kernel(int S, int m_pad, int Hd, float eps, bool bf16, const float* __restrict__ part,
                        const float* __restrict__ residual, const void* __restrict__ gain,
                        float* __restrict__ x_out, void* __restrict__ n_out) {
    __shared__ float s_red[RN_THREADS / 64];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    float ss = 0.f;
    for (int i = tid * 4; i < Hd; i += RN_THREADS * 4) {
        floatx4 v = sum_slices4(part, S, m_pad, m, Hd, i);
        if (residual) v += *reinterpret_cast<const floatx4*>(residual + (size_t)m * Hd + i);
        *reinterpret_cast<floatx4*>(x_out + (size_t)m * Hd + i) = v;
        ss += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
    }
    ss = wave_sumf(ss);
    if (lane == 0) s_red[w] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int j = 0; j < RN_THREADS / 64; ++j) tot += s_red[j];
    const float inv = rsqrtf(tot / (float)Hd + eps);
    for (int i = tid * 4; i < Hd; i += RN_THREADS * 4) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(x_out + (size_t)m * Hd + i);   // this thread's own stores
#pragma unroll
        for (int e = 0; e < 4; ++e) from_float(n_out, (size_t)m * Hd + i + e, v[e] * inv * to_float(gain, i + e, bf16), bf16);
    }
}

// qkv slices -> rotary q into Q[b, row], rotary k and v into the draft tree's K/V rows.
__global__ __launch_bounds__(DL_THREADS)
void qkv_rope_kernel(int S, int m_pad, int d, int F, int k, int Rd, int Hq, int Hkv, int dh, float log2_theta, bool bf16,
                     const float* __restrict__ part, const int* __restrict__ pos,
                     void* __restrict__ Q, void* __restrict__ K_draft, void* __restrict__ V_draft) {
    const int m = blockIdx.x, b = m / F, s = m - b * F;
    const int row = draft_row_of(d, s, k);
    const int Nq = (Hq + 2 * Hkv) * dh, half = dh >> 1;
    const float p = (float)pos[m];
    // work items: the rotary pairs (i, i + dh/2) of the query and key heads, then the value elements
    const int npair = (Hq + Hkv) * half;
    const int u = blockIdx.y * DL_THREADS + threadIdx.x;
    if (u < npair) {
        const int head = u / half, i = u - head * half;
        const float a = sum_slices(part, S, m_pad, m, Nq, head * dh + i);
        const float c = sum_slices(part, S, m_pad, m, Nq, head * dh + i + half);
        const float ang = p * exp2f(-log2_theta * (2.f * i) / (float)dh);
        float sn, cs;
        sincosf(ang, &sn, &cs);
        const float ra = a * cs - c * sn, rc = c * cs + a * sn;
        if (head < Hq) {
            const size_t o = (((size_t)b * Rd + row) * Hq + head) * dh;
            from_float(Q, o + i, ra, bf16);
            from_float(Q, o + i + half, rc, bf16);
        } else {
            const size_t o = (((size_t)b * Rd + row) * Hkv + (head - Hq)) * dh;
            from_float(K_draft, o + i, ra, bf16);
            from_float(K_draft, o + i + half, rc, bf16);
        }
    } else if (u < npair + Hkv * dh) {
        const int e = u - npair;
        from_float(V_draft, ((size_t)b * Rd + row) * Hkv * dh + e, sum_slices(part, S, m_pad, m, Nq, (Hq + Hkv) * dh + e), bf16);
    }
}

// act = silu(gate) * up in the activation type.
__global__ __launch_bounds__(DL_THREADS)
void swiglu_kernel(int S, int m_pad, int inter, bool bf16, const float* __restrict__ part, void* __restrict__ act) {
    const int m = blockIdx.x;
    const int i = blockIdx.y * DL_THREADS + threadIdx.x;
    if (i >= inter) return;
    const float gt = sum_slices(part, S, m_pad, m, 2 * inter, i);
    const float up = sum_slices(part, S, m_pad, m, 2 * inter, inter + i);
    from_float(act, (size_t)m * inter + i, gt / (1.f + __expf(-gt)) * up, bf16);
}

// feature = residual + sum of the slices, into the draft tree's feature rows.
__global__ __launch_bounds__(DL_THREADS)
void feature_out_kernel(int S, int m_pad, int d, int F, int k, int Rd, int Hd, bool bf16, const float* __restrict__ part,
                        const float* __restrict__ residual, void* __restrict__ draft_feature) {
    const int m = blockIdx.x, b = m / F, s = m - b * F;
    const int i = blockIdx.y * DL_THREADS + threadIdx.x;
    if (i >= Hd) return;
    const int row = draft_row_of(d, s, k);
    from_float(draft_feature, ((size_t)b * Rd + row) * Hd + i,
               residual[(size_t)m * Hd + i] + sum_slices(part, S, m_pad, m, Hd, i), bf16);
}

struct ZeroJobs { unsigned* p[4]; size_t n4[4]; };
__global__ __launch_bounds__(DL_THREADS)
void zero_fill_kernel(ZeroJobs z) {                    // one launch clears all four arrays
#pragma unroll
    for (int j = 0; j < 4; ++j)
        for (size_t i = (size_t)blockIdx.x * DL_THREADS + threadIdx.x; i < z.n4[j]; i += (size_t)gridDim.x * DL_THREADS)
            z.p[j][i] = 0u;
}

// ---- host side ---------------------------------------------------------------------------------

static int draft_rows(const eagle2_cfg* c) { const int r = n_draft_rows(c); return r < 2 ? 2 : r; }

// K slices per matrix: as many as keep tasks * slices <= 640 workgroups, at most 32, and every wave of
// every slice at least one 256-byte stage
static int pick_slices(int n_out, int64_t row_bytes) {
    const int ntask = (n_out + DL_ROWS - 1) / DL_ROWS;
    const int stages = (int)(row_bytes / DL_CHUNK);
    int s = 640 / ntask;
    if (s > 32) s = 32;
    if (s > stages / 4) s = stages / 4;
    return s < 1 ? 1 : s;
}

struct DraftWs { size_t x_in, part, x0, h1, nrm, act, q, o, pos, hp, attn, total; };
static DraftWs draft_layout(const eagle2_cfg* cfg, const eagle2_draft_cfg* dc, const eagle2_attn_cfg* ac, const eagle2_cfg* acfg) {
    const size_t M = (size_t)cfg->batch * cfg->topk, m_pad = (M + 15) / 16 * 16, es = elem_size(cfg);
    const size_t Hd = cfg->hidden, Rd = draft_rows(cfg);
    const size_t nq = (size_t)(dc->n_q_heads + 2 * dc->n_kv_heads) * dc->head_dim;
    // largest (slices x outputs) over the five matrices
    const size_t inter = dc->intermediate, qd = (size_t)dc->n_q_heads * dc->head_dim;
    const size_t need[5] = {Hd * pick_slices((int)Hd, 2 * Hd * es), nq * pick_slices((int)nq, Hd * es), Hd * pick_slices((int)Hd, qd * es),
                            2 * inter * pick_slices((int)(2 * inter), Hd * es), Hd * pick_slices((int)Hd, inter * es)};
    size_t pmax = 0;
    for (size_t v : need) pmax = v > pmax ? v : pmax;
    DraftWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += round_up(bytes, 256); return at; };
    w.x_in = take(M * 2 * Hd * es);
    w.part = take(m_pad * pmax * sizeof(float));
    w.x0 = take(M * Hd * sizeof(float));
    w.h1 = take(M * Hd * sizeof(float));
    w.nrm = take(M * Hd * es);
    w.act = take(M * (size_t)dc->intermediate * es);
    w.q = take((size_t)cfg->batch * Rd * dc->n_q_heads * dc->head_dim * es);
    w.o = take((size_t)cfg->batch * Rd * dc->n_q_heads * dc->head_dim * es);
    w.pos = take(M * sizeof(int));
    size_t kmax = 2 * Hd > qd ? 2 * Hd : qd;               // widest input row of the five products
    kmax = kmax > inter ? kmax : inter;
    w.hp = take(M > 16 ? m_pad * kmax * es : 0);           // re-tiled input rows of the many-row path
    size_t aw = attn_workspace_rows(acfg, ac, 1);          // pass 0 has one query row, later passes k
    const size_t aw_k = attn_workspace_rows(acfg, ac, cfg->topk < acfg->n_tree ? cfg->topk : acfg->n_tree);
    w.attn = take(aw > aw_k ? aw : aw_k);
    w.total = o;
    return w;
}

static int validate_draft(const eagle2_cfg* cfg, const eagle2_draft_cfg* dc) {
    E2_REQUIRE(dc != nullptr, EAGLE2_ERR_ARG, "draft cfg is null");
    E2_REQUIRE(dc->head_dim == 64 || dc->head_dim == 128, EAGLE2_ERR_SHAPE, "draft head_dim %d is not 64 or 128", dc->head_dim);
    E2_REQUIRE(dc->n_kv_heads >= 1 && dc->n_q_heads % dc->n_kv_heads == 0 && dc->n_q_heads >= dc->n_kv_heads && dc->n_q_heads <= 1024,
               EAGLE2_ERR_SHAPE, "draft heads %d/%d", dc->n_q_heads, dc->n_kv_heads);
    const int64_t es = elem_size(cfg);
    E2_REQUIRE(dc->intermediate >= 1 && ((int64_t)dc->intermediate * es) % 256 == 0 && (int64_t)dc->intermediate * es >= 1024,
               EAGLE2_ERR_SHAPE, "draft intermediate size %d: a row of the down projection must be a multiple of 256 bytes (>= 1024)",
               dc->intermediate);
    E2_REQUIRE(((int64_t)dc->n_q_heads * dc->head_dim * es) % 256 == 0 && (int64_t)dc->n_q_heads * dc->head_dim * es >= 1024,
               EAGLE2_ERR_SHAPE, "draft n_q_heads*head_dim: a row of the output projection must be a multiple of 256 bytes (>= 1024)");
    E2_REQUIRE(dc->eps > 0.f && dc->rope_theta > 1.f, EAGLE2_ERR_ARG, "draft eps / rope_theta out of range");
    E2_REQUIRE(draft_rows(cfg) <= EAGLE2_MAX_TREE, EAGLE2_ERR_SHAPE, "1 + (depth-1)*topk = %d draft rows exceed %d",
               n_draft_rows(cfg), EAGLE2_MAX_TREE);
    return EAGLE2_OK;
}

// The attention of the draft rows reuses eagle2_tree_attn with the draft tree as the tree.
static void draft_attn_cfgs(const eagle2_cfg* cfg, const eagle2_draft_cfg* dc, int64_t total_prefix,
                            eagle2_cfg* acfg, eagle2_attn_cfg* ac) {
    *acfg = *cfg;
    acfg->n_tree = draft_rows(cfg);
    acfg->flags = 0;
    acfg->static_tree = nullptr;
    ac->n_q_heads = dc->n_q_heads;
    ac->n_kv_heads = dc->n_kv_heads;
    ac->head_dim = dc->head_dim;
    ac->scale = 0.f;
    ac->total_prefix = total_prefix;
}

template <bool BF16>
static int launch_linear(const void* X, int64_t x_seq_bytes, int M, int F, const void* W, int n_out, int64_t row_bytes,
                         float* part, int m_pad, void* hp_ws, int* slices_out, hipStream_t st) {
    if (M > 16) {
        // many rows (batched serving): one pass over W for up to 160 rows instead of one per 16-row block;
        // the output is dense [M, n_out], i.e. a single slice with row pitch n_out
        *slices_out = 1;
        return gemm_rows(BF16, X, x_seq_bytes, M, F, W, n_out, (int)row_bytes, part, hp_ws, nullptr, 0, st);
    }
    const int S = pick_slices(n_out, row_bytes);
    const int ntask = (n_out + DL_ROWS - 1) / DL_ROWS;
    int G = 2 * device_cu_count();
    if (G > ntask) G = ntask;
    dim3 grid(G, m_pad / 16, S);
    hipLaunchKernelGGL((linear_kernel<BF16, false>), grid, dim3(DL_THREADS), 4 * DL_STAGE, st,
                       static_cast<const uint8_t*>(W), (int)row_bytes, n_out,
                       static_cast<const uint8_t*>(X), x_seq_bytes, M, F, part, m_pad, static_cast<void*>(nullptr));
    E2_HIP(hipGetLastError());
    *slices_out = S;
    return EAGLE2_OK;
}

// The gate / up product with the SwiGLU step in its task ends: possible when the product is not split over
// workgroups anyway (enough tasks to fill the machine) and tasks pair whole 32-row blocks.
static bool glu_fusable(int M, int inter, int64_t row_bytes) {
    return M <= 16 && inter % 32 == 0 && pick_slices(2 * inter, row_bytes) == 1;
}
template <bool BF16>
static int launch_linear_glu(const void* X, int64_t x_seq_bytes, int M, const void* Wgu, int inter, int64_t row_bytes,
                             void* act, int m_pad, hipStream_t st) {
    const int ntask = inter / 32;
    int G = 2 * device_cu_count();
    if (G > ntask) G = ntask;
    hipLaunchKernelGGL((linear_kernel<BF16, true>), dim3(G, m_pad / 16, 1), dim3(DL_THREADS), 4 * DL_STAGE, st,
                       static_cast<const uint8_t*>(Wgu), (int)row_bytes, inter,
                       static_cast<const uint8_t*>(X), x_seq_bytes, M, 1, static_cast<float*>(nullptr), m_pad, act);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

}  // namespace eagle2

using namespace eagle2;

extern "C" size_t eagle2_draft_workspace_bytes(const eagle2_cfg* cfg, const eagle2_draft_cfg* dc, int64_t total_prefix) {
    if (validate_cfg(cfg) != EAGLE2_OK || validate_draft(cfg, dc) != EAGLE2_OK) return 0;
    eagle2_cfg acfg;
    eagle2_attn_cfg ac;
    draft_attn_cfgs(cfg, dc, total_prefix, &acfg, &ac);
    if (validate_cfg(&acfg) != EAGLE2_OK || validate_attn(&acfg, &ac) != EAGLE2_OK) return 0;
    return draft_layout(cfg, dc, &ac, &acfg).total;
}

extern "C" int eagle2_draft_forward(const eagle2_cfg* cfg, const eagle2_draft_cfg* dc, const eagle2_draft_weights* wt, int32_t d,
                                    const int32_t* cand_token, const int32_t* cand_parent, const int32_t* frontier,
                                    const int32_t* root_token, const void* root_feature, const int32_t* prefix_len,
                                    const void* K_prefix, const void* V_prefix, const int64_t* kv_offsets, int64_t total_prefix,
                                    void* draft_feature, void* K_draft, void* V_draft, uint64_t* draft_mask,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    rc = validate_draft(cfg, dc);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(d >= 0 && d < cfg->depth, EAGLE2_ERR_ARG, "eagle2_draft_forward: pass index %d outside [0, %d)", d, cfg->depth);
    E2_REQUIRE(wt && wt->embed && wt->fc && wt->g_attn && wt->wqkv && wt->wo && wt->g_mlp && wt->wgu && wt->wdown, EAGLE2_ERR_ARG,
               "eagle2_draft_forward: null weight pointer");
    E2_REQUIRE(cand_token && cand_parent && frontier && root_token && root_feature && prefix_len && kv_offsets &&
               draft_feature && K_draft && V_draft && draft_mask, EAGLE2_ERR_ARG, "eagle2_draft_forward: null pointer argument");
    E2_REQUIRE(aligned16(wt->embed) && aligned16(wt->fc) && aligned16(wt->wqkv) && aligned16(wt->wo) && aligned16(wt->wgu) &&
               aligned16(wt->wdown) && aligned16(draft_feature) && aligned16(K_draft) && aligned16(V_draft) && aligned16(root_feature),
               EAGLE2_ERR_ARG, "eagle2_draft_forward: tensors must be 16-byte aligned");
    eagle2_cfg acfg;
    eagle2_attn_cfg ac;
    draft_attn_cfgs(cfg, dc, total_prefix, &acfg, &ac);
    rc = validate_cfg(&acfg);
    if (rc != EAGLE2_OK) return rc;
    rc = validate_attn(&acfg, &ac);
    if (rc != EAGLE2_OK) return rc;
    const DraftWs L = draft_layout(cfg, dc, &ac, &acfg);
    E2_REQUIRE(workspace && workspace_bytes >= L.total, EAGLE2_ERR_WORKSPACE,
               "eagle2_draft_forward: workspace of %zu bytes, need %zu", workspace_bytes, L.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const bool bf = cfg->dtype == EAGLE2_DTYPE_BF16;
    const int es = elem_size(cfg);
    const int B = cfg->batch, k = cfg->topk, D = cfg->depth, Hd = cfg->hidden, C = n_cand(cfg);
    const int F = d == 0 ? 1 : k, M = B * F, m_pad = (M + 15) / 16 * 16;
    const int Rd = draft_rows(cfg), words = (Rd + 63) / 64;
    const int Hq = dc->n_q_heads, Hkv = dc->n_kv_heads, dh = dc->head_dim, inter = dc->intermediate;
    const int nq = (Hq + 2 * Hkv) * dh;
    void* x_in = ws + L.x_in;
    float* part = reinterpret_cast<float*>(ws + L.part);
    float* x0 = reinterpret_cast<float*>(ws + L.x0);
    float* h1 = reinterpret_cast<float*>(ws + L.h1);
    void* nrm = ws + L.nrm;
    void* act = ws + L.act;
    void* Q = ws + L.q;
    void* O = ws + L.o;
    int* pos = reinterpret_cast<int*>(ws + L.pos);

    if (d == 0) {
        // rows of later passes are keys (masked) and queries (ignored) of this pass's attention: keep them finite
        ZeroJobs z;                                        // every size is a multiple of 4 bytes
        z.p[0] = static_cast<unsigned*>(K_draft);  z.n4[0] = (size_t)B * Rd * Hkv * dh * es / 4;
        z.p[1] = static_cast<unsigned*>(V_draft);  z.n4[1] = z.n4[0];
        z.p[2] = static_cast<unsigned*>(Q);        z.n4[2] = (size_t)B * Rd * Hq * dh * es / 4;
        z.p[3] = reinterpret_cast<unsigned*>(draft_mask);  z.n4[3] = (size_t)B * Rd * words * 2;
        hipLaunchKernelGGL(zero_fill_kernel, dim3(64), dim3(DL_THREADS), 0, st, z);
        E2_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(draft_gather_kernel, dim3(M), dim3(DL_THREADS), 0, st, d, F, k, D, C, Hd, Rd, words, cfg->vocab, bf,
                       cand_token, cand_parent, frontier, root_token, root_feature, prefix_len, wt->embed, draft_feature,
                       reinterpret_cast<unsigned long long*>(draft_mask), x_in, pos);
    E2_HIP(hipGetLastError());
    int S = 1;
#define E2_LIN(X, XSEQ, FF, WT, NOUT, KIN)                                                                         \
    rc = bf ? launch_linear<true>(X, XSEQ, M, FF, WT, NOUT, (int64_t)(KIN) * es, part, m_pad, ws + L.hp, &S, st)              \
            : launch_linear<false>(X, XSEQ, M, FF, WT, NOUT, (int64_t)(KIN) * es, part, m_pad, ws + L.hp, &S, st);            \
    if (rc != EAGLE2_OK) return rc
    // fusion of [embedding ; feature], then the attention block
    E2_LIN(x_in, (int64_t)2 * Hd * es, 1, wt->fc, Hd, 2 * Hd);
    hipLaunchKernelGGL(sum_rmsnorm_kernel, dim3(M), dim3(RN_THREADS), 0, st, S, m_pad, Hd, dc->eps, bf, part,
                       static_cast<const float*>(nullptr), wt->g_attn, x0, nrm);
    E2_LIN(nrm, (int64_t)Hd * es, 1, wt->wqkv, nq, Hd);
    hipLaunchKernelGGL(qkv_rope_kernel, dim3(M, ((Hq + Hkv) * (dh / 2) + Hkv * dh + DL_THREADS - 1) / DL_THREADS), dim3(DL_THREADS), 0, st, S, m_pad, d, F, k, Rd, Hq, Hkv, dh,
                       log2f(dc->rope_theta), bf, part, pos, Q, K_draft, V_draft);
    E2_HIP(hipGetLastError());
    // only this pass's rows are queries; all draft rows are keys (later rows are zero and masked)
    const int row_base = d == 0 ? 0 : 1 + (d - 1) * k;
    rc = tree_attn_rows(&acfg, &ac, row_base, F, Q, K_prefix, V_prefix, nullptr, nullptr, kv_offsets, prefix_len, K_draft, V_draft, draft_mask, O,
                        nullptr, ws + L.attn, L.total - L.attn, stream);
    if (rc != EAGLE2_OK) return rc;
    // output projection reads this pass's rows of O: row (b, s) at O + (b*Rd + row_base + s) * Hq*dh
    E2_LIN(static_cast<const uint8_t*>(O) + (size_t)row_base * Hq * dh * es, (int64_t)Rd * Hq * dh * es, F, wt->wo, Hd, Hq * dh);
    hipLaunchKernelGGL(sum_rmsnorm_kernel, dim3(M), dim3(RN_THREADS), 0, st, S, m_pad, Hd, dc->eps, bf, part, x0, wt->g_mlp, h1, nrm);
    // SwiGLU MLP
    if (glu_fusable(M, inter, (int64_t)Hd * es)) {
        rc = bf ? launch_linear_glu<true>(nrm, (int64_t)Hd * es, M, wt->wgu, inter, (int64_t)Hd * es, act, m_pad, st)
                : launch_linear_glu<false>(nrm, (int64_t)Hd * es, M, wt->wgu, inter, (int64_t)Hd * es, act, m_pad, st);
        if (rc != EAGLE2_OK) return rc;
    } else {
        E2_LIN(nrm, (int64_t)Hd * es, 1, wt->wgu, 2 * inter, Hd);
        hipLaunchKernelGGL(swiglu_kernel, dim3(M, (inter + DL_THREADS - 1) / DL_THREADS), dim3(DL_THREADS), 0, st, S, m_pad, inter, bf, part, act);
    }
    E2_LIN(act, (int64_t)inter * es, 1, wt->wdown, Hd, inter);
    hipLaunchKernelGGL(feature_out_kernel, dim3(M, (Hd + DL_THREADS - 1) / DL_THREADS), dim3(DL_THREADS), 0, st, S, m_pad, d, F, k, Rd,
                       Hd, bf, part, h1, draft_feature);
#undef E2_LIN
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}
