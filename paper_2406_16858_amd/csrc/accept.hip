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
#include <stdlib.h>
#include <mutex>

namespace eagle2 {

constexpr int AM_THREADS = 1024;
constexpr int SAMPLE_WGS = 32;           // most workgroups that cooperate on one sampling sequence
constexpr int SAMPLE_MAXE = 16;          // vocabulary entries a thread can keep in registers
constexpr int SAMPLE_THREADS = 256;
constexpr int SAMPLE_NPART = 4;          // doubles exchanged per workgroup per pass
constexpr int SAMPLE_SLOT = 8;           // 64-bit words per exchange slot: two tagged halves per double
constexpr unsigned SPIN_LIMIT = 1u << 22;
constexpr int SAMPLE_WAVES = SAMPLE_THREADS / 64;
constexpr int SAMPLE_WORDS = 2 * SAMPLE_WGS * SAMPLE_SLOT;   // words of exchange slots per sequence (two sets)

struct AcceptWs { size_t choice, bar, part, total; };
static AcceptWs accept_layout(const eagle2_cfg* cfg) {
    AcceptWs w;
    w.choice = 0;
    w.bar = round_up((size_t)cfg->batch * cfg->n_tree * sizeof(int), 256);
    w.part = w.bar + round_up((size_t)cfg->batch * sizeof(unsigned), 256);
    w.total = w.part + round_up((size_t)cfg->batch * SAMPLE_WORDS * sizeof(unsigned long long), 256);
    return w;
}
size_t accept_workspace(const eagle2_cfg* cfg) { return accept_layout(cfg).total; }

// grid (N, B): arg-max of one row of target logits, lowest id on ties
__global__ __launch_bounds__(AM_THREADS)
void row_argmax_kernel(const float* __restrict__ logits, int V, int N, const int* __restrict__ mode,
                       int* __restrict__ choice, unsigned* __restrict__ fail, int nfail,
                       unsigned long long* __restrict__ slots, int nwords) {
    const int b = blockIdx.y, n = blockIdx.x;
    {   // side job: clear the sampling kernel's failure flags and exchange slots (it runs next)
        const int gid = (blockIdx.y * gridDim.x + blockIdx.x) * AM_THREADS + threadIdx.x;
        const int nth = gridDim.x * gridDim.y * AM_THREADS;
        for (int i = gid; i < nfail; i += nth) fail[i] = 0u;
        for (int i = gid; i < nwords; i += nth) slots[i] = 0ull;
    }
    if (mode[b] != EAGLE2_MODE_GREEDY) return;
    const float* row = logits + ((size_t)b * N + n) * (size_t)V;
    float bv = -INFINITY;
    int bi = INT_MAX;
    if ((V & 3) == 0) {
        const floatx4* r4 = reinterpret_cast<const floatx4*>(row);
        const int n4 = V >> 2;
        // eight independent loads in flight per thread: a row is only a few loads per thread, and taken one
        // at a time they cost a memory round trip each.  Every group is issued whole: a load beyond the row's end
        // re-reads its last piece (and is ignored), so no thread falls back to one load per round trip.
        constexpr int UN = 8;
        for (int i = threadIdx.x; i < n4; i += UN * AM_THREADS) {
            floatx4 x[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int idx = i + u * AM_THREADS;
                x[u] = __builtin_nontemporal_load(r4 + (idx < n4 ? idx : n4 - 1));
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {             // (ids increase with u and e: the strict comparison keeps the lowest)
                const int idx = i + u * AM_THREADS;
                if (idx < n4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) if (x[u][e] > bv) { bv = x[u][e]; bi = idx * 4 + e; }
                }
            }
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

// one wave: follow the matching child from the root
__device__ __forceinline__ void greedy_walk(int b, int lane, int N, int D, const int* __restrict__ choice,
                                            const int* __restrict__ tree_token, const int* __restrict__ tree_parent,
                                            int* __restrict__ accept_len, int* __restrict__ accept_path,
                                            int* __restrict__ bonus) {
    const int* tok = tree_token + (size_t)b * N;
    const int* par = tree_parent + (size_t)b * N;
    const int* ch = choice + (size_t)b * N;
    int* path = accept_path + (size_t)b * (D + 1);
    // each lane keeps its (up to two) rows in registers: N <= 128
    const int c0 = lane, c1 = lane + 64;
    const int p0 = c0 < N ? par[c0] : -2, t0 = c0 < N ? tok[c0] : -1, w0 = c0 < N ? ch[c0] : -1;
    const int p1 = c1 < N ? par[c1] : -2, t1 = c1 < N ? tok[c1] : -1, w1 = c1 < N ? ch[c1] : -1;
    int cur = 0, len = 0;
    if (lane == 0) path[0] = 0;
    for (int step = 0; step < D; ++step) {
        const int want = cur < 64 ? read_lane_dyn(w0, cur) : read_lane_dyn(w1, cur - 64);
        const unsigned long long m0 = __ballot(c0 > cur && p0 == cur && t0 == want);
        const unsigned long long m1 = __ballot(c1 > cur && p1 == cur && t1 == want);
        int found = -1;
        if (m0) found = __ffsll((long long)m0) - 1;
        else if (m1) found = 64 + __ffsll((long long)m1) - 1;
        if (found < 0) break;
        cur = found;
        ++len;
        if (lane == 0) path[len] = cur;
    }
    if (lane == 0) {
        for (int i = len + 1; i <= D; ++i) path[i] = -1;
        accept_len[b] = len;
        bonus[b] = cur < 64 ? read_lane_dyn(w0, cur) : read_lane_dyn(w1, cur - 64);
    }
}

// grid (B), one wave per sequence; used when no sequence can sample
__global__ __launch_bounds__(64)
void greedy_walk_kernel(int N, int D, const int* __restrict__ mode, const int* __restrict__ choice,
                        const int* __restrict__ tree_token, const int* __restrict__ tree_parent,
                        int* __restrict__ accept_len, int* __restrict__ accept_path, int* __restrict__ bonus) {
    if (mode[blockIdx.x] != EAGLE2_MODE_GREEDY) return;
    greedy_walk(blockIdx.x, threadIdx.x, N, D, choice, tree_token, tree_parent, accept_len, accept_path, bonus);
}

// ---- sampling ------------------------------------------------------------------------

struct SampleCtx {
    unsigned* fail;              // this sequence's failure flag
    unsigned long long* slots;   // [2][SAMPLE_WGS][SAMPLE_SLOT]
    int pass;
    int nwg;                     // workgroups cooperating on this sequence (<= SAMPLE_WGS)
};

// All-gather of SAMPLE_NPART doubles among the workgroups of one sequence.  Every 64-bit word
// a workgroup publishes carries half a double plus the pass number (tag << 32 | half), so each
// word validates itself: no flag, no ordering between stores, one store and one load on the
// critical path.  Thread 8*g + j of every workgroup waits for word j of workgroup g's slot and
// drops its half into `out` (LDS, doubles viewed as pairs of 32-bit words).  Slots alternate
// between two sets by pass parity: a workgroup can only be one exchange ahead of the slowest
// one.  The wait is bounded; false means it expired and the kernel gives up cleanly.
__device__ bool exchange(SampleCtx& cx, const double (&mine)[SAMPLE_NPART], double* out /*LDS*/, int* s_ok) {
    const int wg = blockIdx.x, tid = threadIdx.x;
    unsigned long long* buf = cx.slots + (size_t)(cx.pass & 1) * SAMPLE_WGS * SAMPLE_SLOT;
    const unsigned long long tag = ((unsigned long long)cx.pass + 1ull) << 32;
    __syncthreads();                                   // the previous exchange's `out` is no longer read
    if (tid == 0) *s_ok = 1;
    if (tid < SAMPLE_SLOT) {
        const double v = mine[tid >> 1];
        const unsigned half = (tid & 1) ? (unsigned)__double2hiint(v) : (unsigned)__double2loint(v);
        __hip_atomic_store(buf + wg * SAMPLE_SLOT + tid, tag | half, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (tid < cx.nwg * SAMPLE_SLOT) {
        unsigned spins = 0;
        bool ok = true;
        unsigned long long wv;
        // relaxed device-scope loads are served at the coherence point: no cache invalidation per poll
        while (((wv = __hip_atomic_load(buf + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) != (tag >> 32)) {
            __builtin_amdgcn_s_sleep(2);
            if ((++spins & 1023u) == 0u &&
                (spins > SPIN_LIMIT || __hip_atomic_load(cx.fail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                ok = false;
                atomicExch(cx.fail, 1u);
                break;
            }
        }
        if (ok) reinterpret_cast<unsigned*>(out)[tid] = (unsigned)wv;    // slot g word j -> double g*4 + j/2, half j&1
        else *s_ok = 0;
    }
    __syncthreads();
    cx.pass += 1;
    return *s_ok != 0;
}

// The rejection loop's exchange: sums two doubles per wave over all waves of all workgroups of a
// sequence with two barriers.  Every wave drops its pair into s_red; after the first barrier wave 0
// publishes the workgroup's pair (four tagged words, the first half of its slot) and the first
// nwg * 4 threads each wait for one word of one workgroup; after the second barrier every wave adds
// the gathered pairs itself, in the same order everywhere.  *s_ok must be 1 on entry and is cleared
// for good when a bounded wait expires.
__device__ bool exchange_sum2(SampleCtx& cx, double a, double b, double* s_red /*2 per wave*/, double* out /*LDS, 2 per wg*/,
                              int* s_ok, double& ga, double& gb) {
    const int wg = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long* buf = cx.slots + (size_t)(cx.pass & 1) * SAMPLE_WGS * SAMPLE_SLOT;
    const unsigned tagw = (unsigned)cx.pass + 1u;
    if (lane == 0) { s_red[wave * 2] = a; s_red[wave * 2 + 1] = b; }
    __syncthreads();                                   // also: the previous exchange's `out` is no longer read
    if (tid < 4) {
        double v = 0.0;
#pragma unroll
        for (int w = 0; w < SAMPLE_WAVES; ++w) v += s_red[w * 2 + (tid >> 1)];
        const unsigned half = (tid & 1) ? (unsigned)__double2hiint(v) : (unsigned)__double2loint(v);
        __hip_atomic_store(buf + wg * SAMPLE_SLOT + tid, ((unsigned long long)tagw << 32) | half, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < cx.nwg * 4) {
        const unsigned long long* src = buf + (tid >> 2) * SAMPLE_SLOT + (tid & 3);
        unsigned spins = 0;
        bool ok = true;
        unsigned long long wv;
        while (((wv = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) != tagw) {
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 1023u) == 0u &&
                (spins > SPIN_LIMIT || __hip_atomic_load(cx.fail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                ok = false;
                atomicExch(cx.fail, 1u);
                break;
            }
        }
        if (ok) reinterpret_cast<unsigned*>(out)[tid] = (unsigned)wv;     // workgroup g: doubles 2g, 2g + 1
        else *s_ok = 0;
    }
    __syncthreads();
    cx.pass += 1;
    if (*s_ok == 0) return false;
    ga = wave_sum(lane < cx.nwg ? out[lane * 2] : 0.0);
    gb = wave_sum(lane < cx.nwg ? out[lane * 2 + 1] : 0.0);
    return true;
}

__device__ __forceinline__ double block_sum(double v, double* s_red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < SAMPLE_THREADS / 64; ++w) t += s_red[w];
    return t;
}
__device__ __forceinline__ double block_max(double v, double* s_red) {
    v = wave_maxd(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = s_red[0];
#pragma unroll
    for (int w = 1; w < SAMPLE_THREADS / 64; ++w) t = fmax(t, s_red[w]);
    return t;
}
__device__ __forceinline__ void block_max2(double& a, double& b, double* s_red2) {
    a = wave_maxd(a);
    b = wave_maxd(b);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { s_red2[(threadIdx.x >> 6) * 2] = a; s_red2[(threadIdx.x >> 6) * 2 + 1] = b; }
    __syncthreads();
    double ta = s_red2[0], tb = s_red2[1];
#pragma unroll
    for (int w = 1; w < SAMPLE_THREADS / 64; ++w) { ta = fmax(ta, s_red2[w * 2]); tb = fmax(tb, s_red2[w * 2 + 1]); }
    a = ta;
    b = tb;
}
// sums two values per thread over the workgroup with one pair of barriers
__device__ __forceinline__ void block_sum2(double& a, double& b, double* s_red2 /* 2 * waves */) {
    a = wave_sum(a);
    b = wave_sum(b);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { s_red2[(threadIdx.x >> 6) * 2] = a; s_red2[(threadIdx.x >> 6) * 2 + 1] = b; }
    __syncthreads();
    double ta = 0.0, tb = 0.0;
#pragma unroll
    for (int w = 0; w < SAMPLE_THREADS / 64; ++w) { ta += s_red2[w * 2]; tb += s_red2[w * 2 + 1]; }
    a = ta;
    b = tb;
}
// exclusive prefix sum of one value per thread, in thread order
__device__ __forceinline__ double block_exclusive_scan(double v, double* s_red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    double inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double up = __shfl_up(inc, o, 64);
        if (lane >= o) inc += up;
    }
    __syncthreads();
    if (lane == 63) s_red[w] = inc;
    __syncthreads();
    double before = 0.0;
    for (int i = 0; i < w; ++i) before += s_red[i];
    return before + (inc - v);
}

struct NodeScalars {      // everything needed to rebuild (p_j(v), q_j(v)) for any v
    double inv_t, mt, ist, md, isd;          // 1/T, max and 1/sum-exp of the target row; same for the draft row
    int has_q;
    int nrej;
    int rej_tok[EAGLE2_MAX_TOPK + 1];
    double rej_itot[EAGLE2_MAX_TOPK + 1];    // 1 / residual mass of rejection i (0: keep p)
    double rej_iqs[EAGLE2_MAX_TOPK + 1];     // 1 / remaining draft mass of rejection i (0: keep q)
};

__device__ __forceinline__ void initial_state(const NodeScalars& ns, float zt, float zd, double& p, double& q) {
    p = exp((double)zt * ns.inv_t - ns.mt) * ns.ist;
    q = ns.has_q ? exp((double)zd - ns.md) * ns.isd : 0.0;
}
// one rejection: p <- norm(max(0, p - q)); the rejected token leaves q; q renormalised
__device__ __forceinline__ void reject_step(int v, int x, double itot, double iqs, double& p, double& q) {
    const double r = fmax(p - q, 0.0);
    if (itot > 0.0) p = r * itot;
    if (v == x) q = 0.0;
    if (iqs > 0.0) q = q * iqs;
}
__device__ __forceinline__ void element_state(const NodeScalars& ns, int v, float zt, float zd, double& p, double& q) {
    initial_state(ns, zt, zd, p, q);
    for (int i = 0; i < ns.nrej; ++i) reject_step(v, ns.rej_tok[i], ns.rej_itot[i], ns.rej_iqs[i], p, q);
}

// grid (nwg, B).  CACHED: every thread owns at most SAMPLE_MAXE consecutive vocabulary
// entries and keeps their current (p_j, q_j) in registers from pass to pass; otherwise the
// state is rebuilt from the logits and the recorded scalars in every pass.  The (p_j, q_j)
// of the current row's children are tracked in LDS by every workgroup, so a decision
// costs one division.
template <bool CACHED>
__global__ __launch_bounds__(SAMPLE_THREADS)
void sample_accept_kernel(int nwg, int V, int N, int D, int k, int R, const int* __restrict__ mode,
                          const int* __restrict__ choice, const float* __restrict__ target_logits, const float* __restrict__ draft_logits,
                          const float* __restrict__ temperature, const float* __restrict__ u_accept,
                          const float* __restrict__ u_bonus, const int* __restrict__ tree_token,
                          const int* __restrict__ tree_parent, const int* __restrict__ tree_cand,
                          unsigned* __restrict__ fails, unsigned long long* __restrict__ slots,
                          int* __restrict__ accept_len, int* __restrict__ accept_path, int* __restrict__ bonus) {
    const int b = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x;
    if (mode[b] == EAGLE2_MODE_GREEDY) {
        if (wg == 0 && tid < 64)
            greedy_walk(b, tid, N, D, choice, tree_token, tree_parent, accept_len, accept_path, bonus);
        return;
    }
    if (mode[b] != EAGLE2_MODE_SAMPLE) return;
    constexpr int KIDS = EAGLE2_MAX_TOPK + 1;
    __shared__ NodeScalars ns;
    __shared__ double s_all[SAMPLE_WGS * SAMPLE_NPART];
    __shared__ double s_red[2 * (SAMPLE_THREADS / 64)];
    __shared__ double s_g[2];                                   // totals shared by the whole workgroup
    __shared__ double s_pk[KIDS], s_qk[KIDS];                   // current (p, q) at the children's tokens
    __shared__ int s_kids[EAGLE2_MAX_TREE];
    __shared__ int s_par[EAGLE2_MAX_TREE], s_tok[EAGLE2_MAX_TREE];
    __shared__ float s_ua[EAGLE2_MAX_TREE];
    __shared__ float s_ztx[KIDS], s_zdx[KIDS];                  // logits at the children's tokens
    __shared__ int s_last[SAMPLE_THREADS / 64];
    __shared__ int s_nkids, s_ok, s_decision, s_cand;

    SampleCtx cx;
    cx.fail = fails + b;
    cx.slots = slots + (size_t)b * SAMPLE_WORDS;
    cx.pass = 0;
    cx.nwg = nwg;

    const float* ub = u_bonus + (size_t)b * N;
    int* path = accept_path + (size_t)b * (D + 1);
    float T = temperature[b];
    if (!(T > 0.f)) T = 1.f;
    const double inv_t = 1.0 / (double)T;
    for (int c = tid; c < N; c += SAMPLE_THREADS) {
        s_par[c] = tree_parent[(size_t)b * N + c];
        s_tok[c] = tree_token[(size_t)b * N + c];
        s_ua[c] = u_accept[(size_t)b * N + c];
    }

    // this workgroup's slice of the vocabulary and this thread's chunk of it (both contiguous,
    // so prefix sums compose)
    const int per_wg = (V + nwg - 1) / nwg;
    const int v_lo = min(V, wg * per_wg), v_hi = min(V, v_lo + per_wg);
    const int per_th = (v_hi - v_lo + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
    const int t_lo = min(v_hi, v_lo + tid * per_th), t_hi = min(v_hi, t_lo + per_th);

    // every thread's chunk starts on a 16-byte boundary of the (16-byte aligned) logit rows
    const bool vec_ok = CACHED && (V & 3) == 0 && (per_wg & 3) == 0 && (per_th & 3) == 0 && SAMPLE_MAXE % 4 == 0 &&
                        ((reinterpret_cast<size_t>(target_logits) | reinterpret_cast<size_t>(draft_logits)) & 15) == 0;
    double pe[CACHED ? SAMPLE_MAXE : 1], qe[CACHED ? SAMPLE_MAXE : 1];

    int cur = 0, len = 0;
    for (int guard = 0; guard <= N; ++guard) {
        // children of cur in flat order (a parallel compaction over the N <= 128 rows)
        if (tid == 0) s_nkids = 0;
        __syncthreads();
        if (tid < 64) {
            int nk = 0;
            for (int c0 = 0; c0 < N; c0 += 64) {
                const int c = c0 + tid;
                const bool is_kid = c < N && c > cur && s_par[c] == cur;
                const unsigned long long m = __ballot(is_kid);
                if (is_kid) s_kids[nk + __popcll(m & ((1ull << tid) - 1ull))] = c;
                nk += __popcll(m);
            }
            if (tid == 0) s_nkids = nk;
        }
        __syncthreads();
        const int nkids = min(s_nkids, KIDS);
        int drow = 0;
        if (nkids > 0) {                                       // the draft row the children were taken from
            const int cid = tree_cand[(size_t)b * N + s_kids[0]];
            if (cid >= k) { const int layer = 2 + (cid - k) / (k * k); drow = 1 + (layer - 2) * k + ((cid - k) % (k * k)) / k; }
            if (drow < 0 || drow >= R) drow = 0;
        }
        const float* zt_row = target_logits + ((size_t)b * N + cur) * (size_t)V;
        const float* zd_row = draft_logits + ((size_t)b * R + drow) * (size_t)V;
        const bool has_q = nkids > 0;
        if (tid < nkids) {                                     // one latency for all children
            const int x = s_tok[s_kids[tid]];
            const bool okx = x >= 0 && x < V;
            s_ztx[tid] = okx ? zt_row[x] : 0.f;
            s_zdx[tid] = okx ? zd_row[x] : 0.f;
        }

        // pass A: (max, sum-exp) of both rows, merged across workgroups
        float zte[CACHED ? SAMPLE_MAXE : 1], zde[CACHED ? SAMPLE_MAXE : 1];
        double mt = -INFINITY, md = -INFINITY;
        if constexpr (CACHED) {
            if (vec_ok) {                                     // uniform: 16-byte loads, four per row and thread
#pragma unroll
                for (int e4 = 0; e4 < SAMPLE_MAXE / 4; ++e4) {
                    const int v = t_lo + e4 * 4;
                    const bool in = v < t_hi;
                    const floatx4 a = in ? *reinterpret_cast<const floatx4*>(zt_row + v) : floatx4{0.f, 0.f, 0.f, 0.f};
                    const floatx4 c = (in && has_q) ? *reinterpret_cast<const floatx4*>(zd_row + v) : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        zte[e4 * 4 + i] = v + i < t_hi ? a[i] : -INFINITY;
                        zde[e4 * 4 + i] = (v + i < t_hi && has_q) ? c[i] : -INFINITY;
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < SAMPLE_MAXE; ++e) {        // all loads in flight together
                    const int v = t_lo + e;
                    zte[e] = v < t_hi ? zt_row[v] : -INFINITY;
                    zde[e] = (v < t_hi && has_q) ? zd_row[v] : -INFINITY;
                }
            }
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) {
                mt = fmax(mt, (double)zte[e] * inv_t);
                md = fmax(md, (double)zde[e]);
            }
        } else {
            for (int v = t_lo; v < t_hi; ++v) {
                mt = fmax(mt, (double)zt_row[v] * inv_t);
                if (has_q) md = fmax(md, (double)zd_row[v]);
            }
        }
        block_max2(mt, md, s_red);
        double st = 0.0, sd = 0.0;
        if constexpr (CACHED) {
            // the exponentials relative to this workgroup's maxima are kept: the global maxima and the
            // normalisers turn them into probabilities with one multiplication each
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) {
                pe[e] = 0.0;
                qe[e] = 0.0;
                if (t_lo + e < t_hi) {
                    pe[e] = exp((double)zte[e] * inv_t - mt);
                    if (has_q) qe[e] = exp((double)zde[e] - md);
                }
                st += pe[e];
                sd += qe[e];
            }
        } else {
            for (int v = t_lo; v < t_hi; ++v) {
                st += exp((double)zt_row[v] * inv_t - mt);
                if (has_q) sd += exp((double)zd_row[v] - md);
            }
        }
        const double wg_mt = mt, wg_md = md;               // this workgroup's maxima (uniform after block_max2)
        block_sum2(st, sd, s_red);
        {
            const double mine[SAMPLE_NPART] = {mt, st, md, sd};
            if (!exchange(cx, mine, s_all, &s_ok)) break;
        }
        if (tid < 64) {                                        // every workgroup combines the same values the same way
            const bool in = tid < nwg;
            const double m_t = in ? s_all[tid * SAMPLE_NPART] : -INFINITY, s_t = in ? s_all[tid * SAMPLE_NPART + 1] : 0.0;
            const double m_d = in ? s_all[tid * SAMPLE_NPART + 2] : -INFINITY, s_d = in ? s_all[tid * SAMPLE_NPART + 3] : 0.0;
            const double gmt = wave_maxd(m_t), gmd = wave_maxd(m_d);
            const double gst = wave_sum(m_t > -INFINITY ? s_t * exp(m_t - gmt) : 0.0);
            const double gsd = wave_sum(m_d > -INFINITY ? s_d * exp(m_d - gmd) : 0.0);
            if (tid == 0) {
                ns.inv_t = inv_t; ns.mt = gmt; ns.ist = 1.0 / gst; ns.md = gmd; ns.isd = has_q ? 1.0 / gsd : 0.0;
                ns.has_q = has_q ? 1 : 0;
                ns.nrej = 0;
            }
        }
        __syncthreads();
        bool moved = false, failed = false;
        if constexpr (CACHED) {
            // Every wave walks the children on its own: lane c keeps child c's current (p, q) and a
            // decision is read off lane ci, so a rejection costs one exchange (two barriers).
            const double fp = wg_mt > -INFINITY ? exp(wg_mt - ns.mt) * ns.ist : 0.0;
            const double fq = (has_q && wg_md > -INFINITY) ? exp(wg_md - ns.md) * ns.isd : 0.0;
#pragma unroll
            for (int e = 0; e < SAMPLE_MAXE; ++e) { pe[e] *= fp; qe[e] *= fq; }
            const int lane = tid & 63;
            double pk = 0.0, qk = 0.0;
            int xk = -1;
            if (lane < nkids) {
                initial_state(ns, s_ztx[lane], s_zdx[lane], pk, qk);
                xk = s_tok[s_kids[lane]];
            }
            for (int ci = 0; ci < nkids; ++ci) {
                const int c = s_kids[ci];
                const int x = s_tok[c];
                const double pc = read_lane_dyn(pk, ci), qc = read_lane_dyn(qk, ci);
                if (x >= 0 && x < V && (double)s_ua[c] < pc / qc) {
                    cur = c; ++len; moved = true;
                    if (wg == 0 && tid == 0 && len <= D) path[len] = c;
                    break;
                }
                // rejected: residual mass and remaining draft mass
                double tot = 0.0, qs = 0.0;
#pragma unroll
                for (int e = 0; e < SAMPLE_MAXE; ++e) {
                    tot += fmax(pe[e] - qe[e], 0.0);
                    if (t_lo + e != x) qs += qe[e];
                }
                tot = wave_sum(tot);
                qs = wave_sum(qs);
                double gt, gq;
                if (!exchange_sum2(cx, tot, qs, s_red, s_all, &s_ok, gt, gq)) { failed = true; break; }
                const double itot = gt > 0.0 ? 1.0 / gt : 0.0, iqs = gq > 0.0 ? 1.0 / gq : 0.0;
                if (lane < nkids) reject_step(xk, x, itot, iqs, pk, qk);
#pragma unroll
                for (int e = 0; e < SAMPLE_MAXE; ++e) reject_step(t_lo + e, x, itot, iqs, pe[e], qe[e]);
            }
        } else {
            // the state is rebuilt from the logits in every pass; the children's (p, q) live in LDS
            if (tid < nkids) initial_state(ns, s_ztx[tid], s_zdx[tid], s_pk[tid], s_qk[tid]);
            __syncthreads();

            for (int ci = 0; ci < nkids; ++ci) {
                const int c = s_kids[ci];
                const int x = s_tok[c];
                if (tid == 0) s_decision = (x >= 0 && x < V && (double)s_ua[c] < s_pk[ci] / s_qk[ci]) ? 1 : 0;
                __syncthreads();
                if (s_decision) { cur = c; ++len; moved = true; if (wg == 0 && tid == 0 && len <= D) path[len] = c; break; }
                // rejected: residual mass and remaining draft mass
                double tot = 0.0, qs = 0.0;
                for (int v = t_lo; v < t_hi; ++v) {
                    double p, q;
                    element_state(ns, v, zt_row[v], zd_row[v], p, q);
                    tot += fmax(p - q, 0.0);
                    if (v != x) qs += q;
                }
                block_sum2(tot, qs, s_red);
                {
                    const double mine[SAMPLE_NPART] = {tot, qs, 0.0, 0.0};
                    if (!exchange(cx, mine, s_all, &s_ok)) { failed = true; break; }
                }
                if (tid < 64) {
                    const double gt0 = wave_sum(tid < nwg ? s_all[tid * SAMPLE_NPART] : 0.0);
                    const double gq0 = wave_sum(tid < nwg ? s_all[tid * SAMPLE_NPART + 1] : 0.0);
                    if (tid == 0) { s_g[0] = gt0; s_g[1] = gq0; }
                }
                __syncthreads();
                const double gt = s_g[0], gq = s_g[1];
                const double itot = gt > 0.0 ? 1.0 / gt : 0.0, iqs = gq > 0.0 ? 1.0 / gq : 0.0;
                if (tid == 0) {
                    const int j = ns.nrej;
                    ns.rej_tok[j] = x; ns.rej_itot[j] = itot; ns.rej_iqs[j] = iqs;
                    ns.nrej = j + 1;
                }
                if (tid < nkids) reject_step(s_tok[s_kids[tid]], x, itot, iqs, s_pk[tid], s_qk[tid]);
                __syncthreads();
            }
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
        const double th_before = block_exclusive_scan(loc, s_red);
        const double wg_sum = block_sum(loc, s_red);
        {
            const double mine[SAMPLE_NPART] = {wg_sum, 0.0, 0.0, 0.0};
            if (!exchange(cx, mine, s_all, &s_ok)) break;
        }
        // every workgroup finds, from the same sums in the same order, which workgroup's slice
        // holds the crossing; only that one scans its slice and writes the result
        double total = 0.0;
        for (int g = 0; g < nwg; ++g) total += s_all[g * SAMPLE_NPART];
        const double goal = (double)ub[cur] * total;
        int owner = -1, last_nonempty = 0;
        double before = 0.0, run = 0.0;
        for (int g = 0; g < nwg; ++g) {
            const double sg = s_all[g * SAMPLE_NPART];
            if (owner < 0 && run + sg > goal) { owner = g; before = run; }
            if (sg > 0.0) last_nonempty = g;
            run += sg;
        }
        const bool crossing = owner >= 0;
        if (!crossing) owner = last_nonempty;          // goal >= total: take the last token with mass
        if (wg != owner) return;
        if (tid == 0) s_cand = INT_MAX;
        __syncthreads();
        if (crossing) {
            double c = before + th_before;
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
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last_pos = max(last_pos, __shfl_xor(last_pos, o, 64));
        if ((tid & 63) == 0) s_last[tid >> 6] = last_pos;
        __syncthreads();
        if (tid == 0) {
            int lp = -1;
            for (int w2 = 0; w2 < SAMPLE_THREADS / 64; ++w2) lp = max(lp, s_last[w2]);
            int out = s_cand != INT_MAX ? s_cand : lp;   // rounding at a slice edge: last token with mass
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

// Everything eagle2_accept does after its arguments are validated: ws is accept_workspace(cfg) bytes of
// device scratch (arg-max choices, failure flags, exchange slots), whoever owns it.
static int accept_launch(const eagle2_cfg* cfg, const int32_t* mode,
                         const float* target_logits, const float* draft_logits,
                         const float* temperature, const float* u_accept, const float* u_bonus,
                         const int32_t* tree_token, const int32_t* tree_parent, const int32_t* tree_cand,
                         int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token,
                         uint8_t* ws, hipStream_t st) {
    const bool can_sample = draft_logits && temperature && u_accept && u_bonus;
    const AcceptWs L = accept_layout(cfg);
    int* choice = reinterpret_cast<int*>(ws + L.choice);
    unsigned* fails = reinterpret_cast<unsigned*>(ws + L.bar);
    unsigned long long* slots = reinterpret_cast<unsigned long long*>(ws + L.part);
    const int B = cfg->batch, N = cfg->n_tree, V = cfg->vocab, D = cfg->depth;

    const int nwords = can_sample ? B * SAMPLE_WORDS : 0;
    hipLaunchKernelGGL(row_argmax_kernel, dim3(N, B), dim3(AM_THREADS), 0, st, target_logits, V, N, mode, choice,
                       fails, can_sample ? B : 0, slots, nwords);
    E2_HIP(hipGetLastError());
    if (!can_sample) {
        hipLaunchKernelGGL(greedy_walk_kernel, dim3(B), dim3(64), 0, st, N, D, mode, choice, tree_token, tree_parent,
                           accept_len, accept_path, bonus_token);
        E2_HIP(hipGetLastError());
        return EAGLE2_OK;
    }
    // all workgroups of a sequence wait for each other, so they must be resident together
    int nwg = 2 * device_cu_count() / B;
    nwg = nwg > SAMPLE_WGS ? SAMPLE_WGS : (nwg < 1 ? 1 : nwg);
    const int per_wg = (V + nwg - 1) / nwg;
    const bool cached = (per_wg + SAMPLE_THREADS - 1) / SAMPLE_THREADS <= SAMPLE_MAXE;
    if (cached)
        hipLaunchKernelGGL(sample_accept_kernel<true>, dim3(nwg, B), dim3(SAMPLE_THREADS), 0, st,
                           nwg, V, N, D, cfg->topk, n_draft_rows(cfg), mode, choice, target_logits, draft_logits, temperature,
                           u_accept, u_bonus, tree_token, tree_parent, tree_cand, fails, slots,
                           accept_len, accept_path, bonus_token);
    else
        hipLaunchKernelGGL(sample_accept_kernel<false>, dim3(nwg, B), dim3(SAMPLE_THREADS), 0, st,
                           nwg, V, N, D, cfg->topk, n_draft_rows(cfg), mode, choice, target_logits, draft_logits, temperature,
                           u_accept, u_bonus, tree_token, tree_parent, tree_cand, fails, slots,
                           accept_len, accept_path, bonus_token);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

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
    return accept_launch(cfg, mode, target_logits, draft_logits, temperature, u_accept, u_bonus, tree_token, tree_parent,
                         tree_cand, accept_len, accept_path, bonus_token, static_cast<uint8_t*>(workspace),
                         static_cast<hipStream_t>(stream));
}

// ---- the same call for callers that cannot provide (or allocate) a workspace ------------------
// The scratch of eagle2_accept (arg-max choices, failure flags, exchange slots) lives in a device array
// of the library itself.  Each GPU holds its own copy at its own address; the host-side name is only a
// handle for hipGetSymbolAddress, never a device address.
namespace eagle2 {
constexpr int NOALLOC_MAX_BATCH = EAGLE2_ACCEPT_NOALLOC_MAX_BATCH;
constexpr size_t NOALLOC_BYTES =
    ((size_t)NOALLOC_MAX_BATCH * EAGLE2_MAX_TREE * sizeof(int) + 255) / 256 * 256 +
    ((size_t)NOALLOC_MAX_BATCH * sizeof(unsigned) + 255) / 256 * 256 +
    ((size_t)NOALLOC_MAX_BATCH * SAMPLE_WORDS * sizeof(unsigned long long) + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

constexpr int NOALLOC_MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static uint8_t* g_scratch_ptr[NOALLOC_MAX_DEVICES];      // device address of `scratch` on each GPU, resolved once

static int scratch_on_current_device(uint8_t** out) {
    int dev = -1;
    E2_HIP(hipGetDevice(&dev));
    E2_REQUIRE(dev >= 0 && dev < NOALLOC_MAX_DEVICES, EAGLE2_ERR_ARG, "eagle2_accept_noalloc: device %d outside [0, %d)", dev,
               NOALLOC_MAX_DEVICES);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        E2_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        E2_REQUIRE(p != nullptr, EAGLE2_ERR_HIP, "eagle2_accept_noalloc: the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = static_cast<uint8_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return EAGLE2_OK;
}
}  // namespace eagle2

extern "C" size_t eagle2_accept_noalloc_scratch_bytes(void) { return NOALLOC_BYTES; }

extern "C" int eagle2_accept_noalloc(const eagle2_cfg* cfg, const int32_t* mode,
                                     const float* target_logits, const float* draft_logits,
                                     const float* temperature, const float* u_accept, const float* u_bonus,
                                     const int32_t* tree_token, const int32_t* tree_parent, const int32_t* tree_cand,
                                     int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(mode && target_logits && tree_token && tree_parent && tree_cand && accept_len && accept_path && bonus_token,
               EAGLE2_ERR_ARG, "eagle2_accept_noalloc: null pointer argument");
    E2_REQUIRE(aligned16(target_logits), EAGLE2_ERR_ARG, "eagle2_accept_noalloc: target_logits must be 16-byte aligned");
    E2_REQUIRE(cfg->batch <= NOALLOC_MAX_BATCH, EAGLE2_ERR_SHAPE,
               "eagle2_accept_noalloc: batch %d exceeds the %d sequences the built-in scratch holds; use eagle2_accept with a workspace",
               cfg->batch, NOALLOC_MAX_BATCH);
    E2_REQUIRE(accept_workspace(cfg) <= NOALLOC_BYTES, EAGLE2_ERR_SHAPE,
               "eagle2_accept_noalloc: this shape needs %zu bytes of scratch, the built-in array has %zu", accept_workspace(cfg),
               NOALLOC_BYTES);
    uint8_t* ws = nullptr;
    rc = scratch_on_current_device(&ws);
    if (rc != EAGLE2_OK) return rc;
    return accept_launch(cfg, mode, target_logits, draft_logits, temperature, u_accept, u_bonus, tree_token, tree_parent,
                         tree_cand, accept_len, accept_path, bonus_token, ws, static_cast<hipStream_t>(stream));
}
