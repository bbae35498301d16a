// Acceptance (Sections 2.1 and 2.2 of the EAGLE-2 paper).
//
// Greedy sequences: one arg-max per tree row over the target logits (all rows in
// parallel), then a walk from the root that follows the child carrying the chosen token.
//
// Sampling sequences: speculative sampling along the tree, in float64.  The state after
// j rejected siblings, p_j = norm(max(0, p_{j-1} - q_{j-1})) and q_j = q_{j-1} with the
// rejected token removed and renormalised, is never stored: every pass recomputes an
// element's (p_j, q_j) from the two logit rows and the j pairs of scalars (residual mass,
// remaining draft mass) found by the earlier passes.  A pass is one sweep over the
// vocabulary by SAMPLE_WGS workgroups per sequence followed by a device-wide barrier
// among them; all workgroups take the same decisions because they evaluate the same
// scalars with the same arithmetic.

#include "common.h"

namespace eagle2 {

constexpr int AM_THREADS = 256;
constexpr int SAMPLE_WGS = 128;          // most workgroups that cooperate on one sampling sequence
constexpr int SAMPLE_MAXE = 8;           // vocabulary entries a thread can keep in registers
constexpr int SAMPLE_THREADS = 256;
constexpr int SAMPLE_NPART = 4;          // doubles exchanged per workgroup per pass
constexpr unsigned SPIN_LIMIT = 1u << 22;

struct AcceptWs { size_t choice, bar, part, total; };
static AcceptWs accept_layout(const eagle2_cfg* cfg) {
    AcceptWs w;
    w.choice = 0;
    w.bar = round_up((size_t)cfg->batch * cfg->n_tree * sizeof(int), 256);
    w.part = w.bar + round_up((size_t)cfg->batch * 2 * sizeof(unsigned), 256);
    w.total = w.part + round_up((size_t)cfg->batch * 2 * SAMPLE_WGS * SAMPLE_NPART * sizeof(double), 256);
    return w;
}
size_t accept_workspace(const eagle2_cfg* cfg) { return accept_layout(cfg).total; }

__global__ void accept_init_kernel(unsigned* bar, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) bar[i] = 0u;
}

// grid (N, B): arg-max of one row of target logits, lowest id on ties
__global__ __launch_bounds__(AM_THREADS)
void row_argmax_kernel(const float* __restrict__ logits, int V, int N, const int* __restrict__ mode,
                       int* __restrict__ choice) {
    const int b = blockIdx.y, n = blockIdx.x;
    if (mode[b] != EAGLE2_MODE_GREEDY) return;
    const float* row = logits + ((size_t)b * N + n) * (size_t)V;
    float bv = -INFINITY;
    int bi = INT_MAX;
    if ((V & 3) == 0) {
        const floatx4* r4 = reinterpret_cast<const floatx4*>(row);
        for (int i = threadIdx.x; i < (V >> 2); i += AM_THREADS) {
            const floatx4 x = r4[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) if (x[e] > bv) { bv = x[e]; bi = i * 4 + e; }
        }
    } else {
        for (int i = threadIdx.x; i < V; i += AM_THREADS) if (row[i] > bv) { bv = row[i]; bi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ranks_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    __shared__ float sv[AM_THREADS / 64];
    __shared__ int si[AM_THREADS / 64];
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < AM_THREADS / 64; ++w)
            if (ranks_before(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
        choice[(size_t)b * N + n] = bi == INT_MAX ? 0 : bi;
    }
}

// grid (B), one wave: follow the matching child from the root
__global__ __launch_bounds__(64)
void greedy_walk_kernel(int N, int D, const int* __restrict__ mode, const int* __restrict__ choice,
                        const int* __restrict__ tree_token, const int* __restrict__ tree_parent,
                        int* __restrict__ accept_len, int* __restrict__ accept_path, int* __restrict__ bonus) {
    const int b = blockIdx.x, lane = threadIdx.x;
    if (mode[b] != EAGLE2_MODE_GREEDY) return;
    const int* tok = tree_token + (size_t)b * N;
    const int* par = tree_parent + (size_t)b * N;
    const int* ch = choice + (size_t)b * N;
    int* path = accept_path + (size_t)b * (D + 1);
    int cur = 0, len = 0;
    if (lane == 0) path[0] = 0;
    for (int step = 0; step < D; ++step) {
        const int want = ch[cur];
        int found = INT_MAX;
        for (int c = lane; c < N; c += 64)
            if (c > cur && par[c] == cur && tok[c] == want) { found = c; break; }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) found = min(found, __shfl_xor(found, o, 64));
        if (found == INT_MAX) break;
        cur = found;
        ++len;
        if (lane == 0) path[len] = cur;
    }
    if (lane == 0) {
        for (int i = len + 1; i <= D; ++i) path[i] = -1;
        accept_len[b] = len;
        bonus[b] = ch[cur];
    }
}

// ---- sampling ------------------------------------------------------------------------

struct SampleCtx {
    unsigned* bar;       // this sequence's barrier counter (monotonic)
    unsigned* fail;      // this sequence's failure flag
    double* part;        // [2][SAMPLE_WGS][SAMPLE_NPART]
    unsigned target;     // arrivals expected at the next barrier
    int pass;
    int nwg;             // workgroups cooperating on this sequence (<= SAMPLE_WGS)
};

// Publishes up to SAMPLE_NPART doubles of this workgroup, waits for all workgroups of the
// sequence, and returns with `out[g*NPART + i]` (LDS) holding every workgroup's values.
// Returns false if the bounded wait expired (then the kernel gives up cleanly).
__device__ bool exchange(SampleCtx& cx, const double (&mine)[SAMPLE_NPART], double* out /*LDS*/, int* s_ok) {
    const int wg = blockIdx.x;
    double* buf = cx.part + (size_t)(cx.pass & 1) * SAMPLE_WGS * SAMPLE_NPART;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 0; i < SAMPLE_NPART; ++i) buf[wg * SAMPLE_NPART + i] = mine[i];
        __threadfence();
        atomicAdd(cx.bar, 1u);
        cx.target += (unsigned)cx.nwg;
        unsigned spins = 0;
        bool ok = true;
        while (__hip_atomic_load(cx.bar, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < cx.target) {
            __builtin_amdgcn_s_sleep(4);
            if (++spins > SPIN_LIMIT || __hip_atomic_load(cx.fail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                ok = false;
                atomicExch(cx.fail, 1u);
                break;
            }
        }
        __threadfence();
        *s_ok = ok ? 1 : 0;
    }
    __syncthreads();
    const bool ok = *s_ok != 0;
    if (ok) {
        for (int i = threadIdx.x; i < cx.nwg * SAMPLE_NPART; i += SAMPLE_THREADS)
            out[i] = __hip_atomic_load(buf + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    cx.pass += 1;
    return ok;
}

__device__ __forceinline__ double block_sum(double v, double* s_red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < SAMPLE_THREADS / 64; ++w) t += s_red[w];
    return t;
}
__device__ __forceinline__ double block_max(double v, double* s_red) {
    v = wave_maxd(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = s_red[0];
    for (int w = 1; w < SAMPLE_THREADS / 64; ++w) t = fmax(t, s_red[w]);
    return t;
}

struct NodeScalars {      // everything needed to rebuild (p_j(v), q_j(v)) for any v
    double inv_t, mt, st, md, sd;
    int has_q;
    int nrej;
    int rej_tok[EAGLE2_MAX_TOPK + 1];
    double rej_tot[EAGLE2_MAX_TOPK + 1];
    double rej_qs[EAGLE2_MAX_TOPK + 1];
};

__device__ __forceinline__ void element_state(const NodeScalars& ns, int v, float zt, float zd, double& p, double& q) {
    p = exp((double)zt * ns.inv_t - ns.mt) / ns.st;
    q = ns.has_q ? exp((double)zd - ns.md) / ns.sd : 0.0;
    for (int i = 0; i < ns.nrej; ++i) {
        const double r = fmax(p - q, 0.0);
        if (ns.rej_tot[i] > 0.0) p = r / ns.rej_tot[i];
        if (v == ns.rej_tok[i]) q = 0.0;
        if (ns.rej_qs[i] > 0.0) q = q / ns.rej_qs[i];
    }
}

// grid (nwg, B).  CACHED: every thread owns at most SAMPLE_MAXE consecutive vocabulary
// entries and keeps their current (p_j, q_j) in registers from pass to pass; otherwise the
// state is rebuilt from the logits and the recorded scalars in every pass.
template <bool CACHED>
__global__ __launch_bounds__(SAMPLE_THREADS)
void sample_accept_kernel(int nwg, int V, int N, int D, int k, int R, const int* __restrict__ mode,
                          const float* __restrict__ target_logits, const float* __restrict__ draft_logits,
                          const float* __restrict__ temperature, const float* __restrict__ u_accept,
                          const float* __restrict__ u_bonus, const int* __restrict__ tree_token,
                          const int* __restrict__ tree_parent, const int* __restrict__ tree_cand,
                          unsigned* __restrict__ bars, double* __restrict__ parts,
                          int* __restrict__ accept_len, int* __restrict__ accept_path, int* __restrict__ bonus) {
    const int b = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x;
    if (mode[b] != EAGLE2_MODE_SAMPLE) return;
    __shared__ NodeScalars ns;
    __shared__ double s_all[SAMPLE_WGS * SAMPLE_NPART];
    __shared__ double s_red[SAMPLE_THREADS / 64];
    __shared__ double s_scan[SAMPLE_THREADS];
    __shared__ int s_kids[EAGLE2_MAX_TREE];
    __shared__ int s_last[SAMPLE_THREADS / 64];
    __shared__ int s_nkids, s_ok, s_decision, s_cand;

    SampleCtx cx;
    cx.bar = bars + (size_t)b * 2;
    cx.fail = bars + (size_t)b * 2 + 1;
    cx.part = parts + (size_t)b * 2 * SAMPLE_WGS * SAMPLE_NPART;
    cx.target = 0;
    cx.pass = 0;
    cx.nwg = nwg;

    const int* tok = tree_token + (size_t)b * N;
    const int* par = tree_parent + (size_t)b * N;
    const int* cnd = tree_cand + (size_t)b * N;
    const float* ua = u_accept + (size_t)b * N;
    const float* ub = u_bonus + (size_t)b * N;
    int* path = accept_path + (size_t)b * (D + 1);
    float T = temperature[b];
    if (!(T > 0.f)) T = 1.f;
    const double inv_t = 1.0 / (double)T;

    // this workgroup's slice of the vocabulary and this thread's chunk of it (both contiguous,
    // so prefix sums compose)
    const int per_wg = (V + nwg - 1) / nwg;
    const int v_lo = min(V, wg * per_wg), v_hi = min(V, v_lo + per_wg);
    const int per_th = (v_hi - v_lo + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
    const int t_lo = min(v_hi, v_lo + tid * per_th), t_hi = min(v_hi, t_lo + per_th);

    double pe[CACHED ? SAMPLE_MAXE : 1], qe[CACHED ? SAMPLE_MAXE : 1];

    int cur = 0, len = 0;
    for (int guard = 0; guard <= N; ++guard) {
        // children of cur in flat order and the draft row they were taken from
        if (tid == 0) {
            int nk = 0;
            for (int c = cur + 1; c < N; ++c) if (par[c] == cur) s_kids[nk++] = c;
            s_nkids = nk;
        }
        __syncthreads();
        const int nkids = s_nkids;
        int drow = 0;
        if (nkids > 0) {
            const int cid = cnd[s_kids[0]];
            if (cid >= k) { const int layer = 2 + (cid - k) / (k * k); drow = 1 + (layer - 2) * k + ((cid - k) % (k * k)) / k; }
            if (drow < 0 || drow >= R) drow = 0;
        }
        const float* zt_row = target_logits + ((size_t)b * N + cur) * (size_t)V;
        const float* zd_row = draft_logits + ((size_t)b * R + drow) * (size_t)V;
        const bool has_q = nkids > 0;

        // pass A: (max, sum-exp) of both rows, merged across workgroups
        double mt = -INFINITY, md = -INFINITY;
        for (int v = t_lo; v < t_hi; ++v) {
            mt = fmax(mt, (double)zt_row[v] * inv_t);
            if (has_q) md = fmax(md, (double)zd_row[v]);
        }
        mt = block_max(mt, s_red);
        md = block_max(md, s_red);
        double st = 0.0, sd = 0.0;
        for (int v = t_lo; v < t_hi; ++v) {
            st += exp((double)zt_row[v] * inv_t - mt);
            if (has_q) sd += exp((double)zd_row[v] - md);
        }
        st = block_sum(st, s_red);
        sd = block_sum(sd, s_red);
        {
            const double mine[SAMPLE_NPART] = {mt, st, md, sd};
            if (!exchange(cx, mine, s_all, &s_ok)) break;
        }
        if (tid == 0) {
            double gmt = -INFINITY, gmd = -INFINITY;
            for (int g = 0; g < nwg; ++g) { gmt = fmax(gmt, s_all[g * SAMPLE_NPART]); gmd = fmax(gmd, s_all[g * SAMPLE_NPART + 2]); }
            double gst = 0.0, gsd = 0.0;
            for (int g = 0; g < nwg; ++g) {
                if (s_all[g * SAMPLE_NPART] > -INFINITY) gst += s_all[g * SAMPLE_NPART + 1] * exp(s_all[g * SAMPLE_NPART] - gmt);
                if (s_all[g * SAMPLE_NPART + 2] > -INFINITY) gsd += s_all[g * SAMPLE_NPART + 3] * exp(s_all[g * SAMPLE_NPART + 2] - gmd);
            }
            ns.inv_t = inv_t; ns.mt = gmt; ns.st = gst; ns.md = gmd; ns.sd = gsd;
            ns.has_q = has_q ? 1 : 0;
            ns.nrej = 0;
        }
        __syncthreads();
        if constexpr (CACHED) {
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) {
                const int v = t_lo + e;
                if (v < t_hi) element_state(ns, v, zt_row[v], has_q ? zd_row[v] : 0.f, pe[e], qe[e]);
                else { pe[e] = 0.0; qe[e] = 0.0; }
            }
        }

        bool moved = false, failed = false;
        for (int ci = 0; has_q && ci < nkids && ci < EAGLE2_MAX_TOPK + 1; ++ci) {
            const int c = s_kids[ci];
            const int x = tok[c];
            if (tid == 0) {
                int dec = 0;
                if (x >= 0 && x < V) {
                    double p, q;
                    element_state(ns, x, zt_row[x], zd_row[x], p, q);
                    dec = ((double)ua[c] < p / q) ? 1 : 0;
                }
                s_decision = dec;
            }
            __syncthreads();
            if (s_decision) { cur = c; ++len; moved = true; if (wg == 0 && tid == 0 && len <= D) path[len] = c; break; }
            // rejected: residual mass and remaining draft mass
            double tot = 0.0, qs = 0.0;
            if constexpr (CACHED) {
#pragma unroll
                for (int e = 0; e < SAMPLE_MAXE; ++e) {
                    tot += fmax(pe[e] - qe[e], 0.0);
                    if (t_lo + e != x) qs += qe[e];
                }
            } else {
                for (int v = t_lo; v < t_hi; ++v) {
                    double p, q;
                    element_state(ns, v, zt_row[v], zd_row[v], p, q);
                    tot += fmax(p - q, 0.0);
                    if (v != x) qs += q;
                }
            }
            tot = block_sum(tot, s_red);
            qs = block_sum(qs, s_red);
            {
                const double mine[SAMPLE_NPART] = {tot, qs, 0.0, 0.0};
                if (!exchange(cx, mine, s_all, &s_ok)) { failed = true; break; }
            }
            double gt = 0.0, gq = 0.0;
            for (int g = 0; g < nwg; ++g) { gt += s_all[g * SAMPLE_NPART]; gq += s_all[g * SAMPLE_NPART + 1]; }
            if (tid == 0) {
                const int j = ns.nrej;
                ns.rej_tok[j] = x; ns.rej_tot[j] = gt; ns.rej_qs[j] = gq;
                ns.nrej = j + 1;
            }
            if constexpr (CACHED) {
#pragma unroll
                for (int e = 0; e < SAMPLE_MAXE; ++e) {
                    const double r = fmax(pe[e] - qe[e], 0.0);
                    if (gt > 0.0) pe[e] = r / gt;
                    if (t_lo + e == x) qe[e] = 0.0;
                    if (gq > 0.0) qe[e] = qe[e] / gq;
                }
            }
            __syncthreads();
        }
        if (failed) break;
        if (moved) continue;

        // no child accepted: draw the emitted token from the current p by inverse CDF
        double loc = 0.0;
        int last_pos = -1;
        if constexpr (CACHED) {
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) { loc += pe[e]; if (pe[e] > 0.0) last_pos = t_lo + e; }
        } else {
            for (int v = t_lo; v < t_hi; ++v) {
                double p, q;
                element_state(ns, v, zt_row[v], has_q ? zd_row[v] : 0.f, p, q);
                loc += p;
                if (p > 0.0) last_pos = v;
            }
        }
        s_scan[tid] = loc;
        const double wg_sum = block_sum(loc, s_red);
        {
            const double mine[SAMPLE_NPART] = {wg_sum, 0.0, 0.0, 0.0};
            if (!exchange(cx, mine, s_all, &s_ok)) break;
        }
        double total = 0.0, before = 0.0;
        for (int g = 0; g < nwg; ++g) { if (g == wg) before = total; total += s_all[g * SAMPLE_NPART]; }
        const double goal = (double)ub[cur] * total;
        if (tid == 0) s_cand = INT_MAX;
        __syncthreads();
        double c = before;
        for (int t = 0; t < tid; ++t) c += s_scan[t];
        // every thread scans its chunk; the smallest index whose running sum passes the goal wins
        if constexpr (CACHED) {
            bool hit = false;
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) {
                c += pe[e];
                if (!hit && t_lo + e < t_hi && c > goal) { atomicMin(&s_cand, t_lo + e); hit = true; }
            }
        } else {
            for (int v = t_lo; v < t_hi; ++v) {
                double p, q;
                element_state(ns, v, zt_row[v], has_q ? zd_row[v] : 0.f, p, q);
                c += p;
                if (c > goal) { atomicMin(&s_cand, v); break; }
            }
        }
        // last token with positive mass, for the (measure-zero) case of no crossing
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last_pos = max(last_pos, __shfl_xor(last_pos, o, 64));
        if ((tid & 63) == 0) s_last[tid >> 6] = last_pos;
        __syncthreads();
        {
            int lp = -1;
            for (int w2 = 0; w2 < SAMPLE_THREADS / 64; ++w2) lp = max(lp, s_last[w2]);
            const double mine[SAMPLE_NPART] = {(double)s_cand, (double)lp, 0.0, 0.0};
            if (!exchange(cx, mine, s_all, &s_ok)) break;
        }
        if (wg == 0 && tid == 0) {
            double best = (double)INT_MAX, lastp = -1.0;
            for (int g = 0; g < nwg; ++g) { best = fmin(best, s_all[g * SAMPLE_NPART]); lastp = fmax(lastp, s_all[g * SAMPLE_NPART + 1]); }
            int out = best < (double)INT_MAX ? (int)best : (int)lastp;
            if (out < 0) out = 0;
            bonus[b] = out;
            accept_len[b] = len;
            path[0] = 0;
            for (int i = len + 1; i <= D; ++i) path[i] = -1;
        }
        return;
    }
    // only reached when the bounded wait expired or the tree was malformed
    if (wg == 0 && tid == 0) { accept_len[b] = -1; bonus[b] = -1; for (int i = 0; i <= D; ++i) path[i] = -1; }
}

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_accept(const eagle2_cfg* cfg, const int32_t* mode,
                             const float* target_logits, const float* draft_logits,
                             const float* temperature, const float* u_accept, const float* u_bonus,
                             const int32_t* tree_token, const int32_t* tree_parent, const int32_t* tree_cand,
                             int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token,
                             void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(mode && target_logits && tree_token && tree_parent && tree_cand && accept_len && accept_path && bonus_token,
               EAGLE2_ERR_ARG, "eagle2_accept: null pointer argument");
    E2_REQUIRE(aligned16(target_logits), EAGLE2_ERR_ARG, "eagle2_accept: target_logits must be 16-byte aligned");
    E2_REQUIRE(workspace && workspace_bytes >= accept_workspace(cfg), EAGLE2_ERR_WORKSPACE,
               "eagle2_accept: workspace of %zu bytes, need %zu", workspace_bytes, accept_workspace(cfg));
    const bool can_sample = draft_logits && temperature && u_accept && u_bonus;
    const AcceptWs L = accept_layout(cfg);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    int* choice = reinterpret_cast<int*>(ws + L.choice);
    unsigned* bars = reinterpret_cast<unsigned*>(ws + L.bar);
    double* parts = reinterpret_cast<double*>(ws + L.part);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = cfg->batch, N = cfg->n_tree, V = cfg->vocab, D = cfg->depth;

    hipLaunchKernelGGL(row_argmax_kernel, dim3(N, B), dim3(AM_THREADS), 0, st, target_logits, V, N, mode, choice);
    E2_HIP(hipGetLastError());
    hipLaunchKernelGGL(greedy_walk_kernel, dim3(B), dim3(64), 0, st, N, D, mode, choice, tree_token, tree_parent,
                       accept_len, accept_path, bonus_token);
    E2_HIP(hipGetLastError());
    if (can_sample) {
        hipLaunchKernelGGL(accept_init_kernel, dim3((2 * B + 255) / 256), dim3(256), 0, st, bars, 2 * B);
        E2_HIP(hipGetLastError());
        // all workgroups of a sequence wait for each other, so they must be resident together
        int nwg = 2 * device_cu_count() / B;
        nwg = nwg > SAMPLE_WGS ? SAMPLE_WGS : (nwg < 1 ? 1 : nwg);
        const int per_wg = (V + nwg - 1) / nwg;
        const bool cached = (per_wg + SAMPLE_THREADS - 1) / SAMPLE_THREADS <= SAMPLE_MAXE;
        if (cached)
            hipLaunchKernelGGL(sample_accept_kernel<true>, dim3(nwg, B), dim3(SAMPLE_THREADS), 0, st,
                               nwg, V, N, D, cfg->topk, n_draft_rows(cfg), mode, target_logits, draft_logits, temperature,
                               u_accept, u_bonus, tree_token, tree_parent, tree_cand, bars, parts,
                               accept_len, accept_path, bonus_token);
        else
            hipLaunchKernelGGL(sample_accept_kernel<false>, dim3(nwg, B), dim3(SAMPLE_THREADS), 0, st,
                               nwg, V, N, D, cfg->topk, n_draft_rows(cfg), mode, target_logits, draft_logits, temperature,
                               u_accept, u_bonus, tree_token, tree_parent, tree_cand, bars, parts,
                               accept_len, accept_path, bonus_token);
        E2_HIP(hipGetLastError());
    }
    return EAGLE2_OK;
}
