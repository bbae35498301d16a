// Reranking phase and flattening (Section 4.2 of the EAGLE-2 paper): global top-(N-1)
// of all candidates by joint score (ties to the lower id, i.e. the shallower node),
// flattening in increasing id order behind the root, parent rows, depths, position ids
// and the ancestor bitmask ("each token can only see its ancestor nodes").
//
// One workgroup per sequence.  The C <= 2048 candidates are ranked by counting (runs of 64
// ranked with lane broadcasts, run against run by binary search); the rest is a handful of
// LDS look-ups.

#include "common.h"

namespace eagle2 {

constexpr int RR_THREADS = 1024;

__global__ __launch_bounds__(RR_THREADS)
void rerank_kernel(int C, int N, int k, int D, int words, int flags,
                   const int* __restrict__ cand_token, const double* __restrict__ cand_score,
                   const int* __restrict__ cand_parent, const int* __restrict__ frontier,
                   const int* __restrict__ static_tree, const int* __restrict__ root_token,
                   const int* __restrict__ prefix_len,
                   int* __restrict__ tree_token, int* __restrict__ tree_parent, int* __restrict__ tree_depth,
                   int* __restrict__ tree_cand, int* __restrict__ position_ids,
                   unsigned long long* __restrict__ mask_bits) {
    __shared__ double s_key[EAGLE2_MAX_CAND];
    __shared__ int s_id[EAGLE2_MAX_CAND];
    __shared__ int s_in[EAGLE2_MAX_CAND];          // rank inside the candidate's own run
    __shared__ int s_rank[EAGLE2_MAX_CAND];
    __shared__ int s_row_of[EAGLE2_MAX_CAND];      // flat row of a candidate, -1 if not selected
    __shared__ int s_sel[EAGLE2_MAX_TREE];         // selected candidate ids (sorted order)
    __shared__ int s_par[EAGLE2_MAX_TREE];         // flat parent row per flat row
    const int b = blockIdx.x, tid = threadIdx.x;
    const double* score = cand_score + (size_t)b * C;
    const int* ctok = cand_token + (size_t)b * C;
    const int* cpar = cand_parent + (size_t)b * C;

    const int nsel = N - 1;
    if (flags & EAGLE2_FLAG_STATIC_TREE) {
        // Section 2.2: a fixed shape whose positions the drafting phase has filled in
        for (int i = tid; i < C; i += RR_THREADS) s_row_of[i] = -1;
        for (int i = tid; i < nsel; i += RR_THREADS) {
            int c = static_tree[i];
            if (c < 0 || c >= C) c = 0;                   // a malformed shape stays in bounds
            s_sel[i] = c;
        }
        __syncthreads();
    } else if (flags & EAGLE2_FLAG_NO_RERANK) {
        // Section 5.2, "w/o reranking": the draft is what the expansion phase selected, i.e. the
        // frontiers of layers 1..D-1 and the k best nodes of layer D (nsel = D*k, checked by the host).
        const int last = k + (D - 2) * k * k;            // first id of layer D (D >= 2 here; D = 1 has no frontier rows)
        for (int i = tid; i < C; i += RR_THREADS) s_row_of[i] = -1;
        for (int i = tid; i < (D - 1) * k; i += RR_THREADS) {
            int c = frontier[((size_t)b * D + 1) * k + i];
            if (c < 0 || c >= C) c = 0;                   // garbage in the caller's frontier stays in bounds
            s_sel[i] = c;
        }
        const int nl = D == 1 ? k : k * k;               // size of layer D
        const int lbase = D == 1 ? 0 : last;
        if (tid < nl) {
            const int c = lbase + tid;
            double key = score[c];
            if ((flags & EAGLE2_FLAG_RANK_BY_CONFIDENCE) && cpar[c] >= 0 && cpar[c] < C) key -= score[cpar[c]];
            s_key[tid] = key;
        }
        __syncthreads();
        if (tid < nl) {
            const double v = s_key[tid];
            int r = 0;
            for (int j = 0; j < nl; ++j) r += ranks_before(s_key[j], j, v, tid) ? 1 : 0;
            if (r < k) s_sel[(D - 1) * k + r] = lbase + tid;
        }
        __syncthreads();
    } else {
    // Rank of every candidate = number of candidates that precede it (score desc, id asc).
    // Candidates are cut into runs of 64.  Inside a run the count is taken with v_readlane
    // broadcasts (no LDS); the run is then laid out sorted in LDS, and the count against every
    // other run is a binary search in that run.
    const int nrun = (C + 63) >> 6;
    const int lane = tid & 63, wave = tid >> 6;
    for (int run = wave; run < nrun; run += RR_THREADS / 64) {
        const int i = run * 64 + lane;
        const double v = i < C ? score[i] : -INFINITY;
        const int id = i < C ? i : INT_MAX;
        int r = 0;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            const double vj = read_lane(v, j);
            r += ((vj > v) | ((vj == v) & (j < lane))) ? 1 : 0;   // same run: id order = lane order (bitwise: no branches)
        }
        s_key[run * 64 + r] = v;
        s_id[run * 64 + r] = id;
        if (i < C) s_in[i] = r;                                   // padding entries sort after the real ones
    }
    __syncthreads();
    for (int i = tid; i < C; i += RR_THREADS) {
        const double v = score[i];
        const int myrun = i >> 6;
        int r = s_in[i];
        for (int run = 0; run < nrun; ++run) {
            if (run == myrun) continue;
            const double* kk = s_key + run * 64;
            const int* ii = s_id + run * 64;
            int lo = 0;                                           // entries [0, lo) precede (v, i)
#pragma unroll
            for (int step = 32; step > 0; step >>= 1)
                if (ranks_before(kk[lo + step - 1], ii[lo + step - 1], v, i)) lo += step;
            if (lo == 63 && ranks_before(kk[63], ii[63], v, i)) lo = 64;
            r += lo;
        }
        s_rank[i] = r;
        s_row_of[i] = -1;
    }
    __syncthreads();
    for (int i = tid; i < C; i += RR_THREADS)
        if (s_rank[i] < nsel) s_sel[s_rank[i]] = i;
    __syncthreads();
    }
    int my_row = -1, my_id = -1;
    if (tid < nsel) {
        my_id = s_sel[tid];
        int below = 0;
        for (int j = 0; j < nsel; ++j) below += s_sel[j] < my_id ? 1 : 0;
        my_row = 1 + below;                          // flat order = increasing candidate id
        if (my_id >= 0 && my_id < C) s_row_of[my_id] = my_row;
    }
    __syncthreads();
    const size_t ob = (size_t)b * N;
    if (tid < nsel && my_id >= 0 && my_id < C) {
        const int par = cpar[my_id];
        const int prow = par < 0 ? 0 : (par < C ? s_row_of[par] : -1);
        const int depth = my_id < k ? 1 : 2 + (my_id - k) / (k * k);
        s_par[my_row] = prow;
        tree_token[ob + my_row] = ctok[my_id];
        tree_parent[ob + my_row] = prow;
        tree_depth[ob + my_row] = depth;
        tree_cand[ob + my_row] = my_id;
        position_ids[ob + my_row] = prefix_len[b] + depth;
    }
    if (tid == 0) {
        s_par[0] = -1;
        tree_token[ob] = root_token[b];
        tree_parent[ob] = -1;
        tree_depth[ob] = 0;
        tree_cand[ob] = -1;
        position_ids[ob] = prefix_len[b];
    }
    __syncthreads();
    if (tid < N) {
        unsigned long long wbits[EAGLE2_MAX_TREE / 64] = {0ull, 0ull};
        int cur = tid;
        for (int step = 0; step < N && cur >= 0; ++step) {   // a path has at most N rows
            wbits[cur >> 6] |= 1ull << (cur & 63);
            const int p = s_par[cur];
            cur = p < cur ? p : -1;                 // parents precede children; stops on bad input
        }
        for (int wi = 0; wi < words; ++wi) mask_bits[(ob + tid) * words + wi] = wbits[wi];
    }
}

size_t rerank_workspace(const eagle2_cfg*) { return 0; }

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_rerank(const eagle2_cfg* cfg,
                             const int32_t* cand_token, const double* cand_score, const int32_t* cand_parent,
                             const int32_t* frontier, const int32_t* root_token, const int32_t* prefix_len,
                             int32_t* tree_token, int32_t* tree_parent, int32_t* tree_depth,
                             int32_t* tree_cand, int32_t* position_ids, uint64_t* mask_bits,
                             void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(cand_token && cand_score && cand_parent && root_token && prefix_len && tree_token && tree_parent &&
               tree_depth && tree_cand && position_ids && mask_bits, EAGLE2_ERR_ARG, "eagle2_rerank: null pointer argument");
    E2_REQUIRE(frontier || !(cfg->flags & EAGLE2_FLAG_NO_RERANK), EAGLE2_ERR_ARG,
               "eagle2_rerank: EAGLE2_FLAG_NO_RERANK needs the frontier array");
    const int C = n_cand(cfg);
    const int words = (cfg->n_tree + 63) / 64;
    hipLaunchKernelGGL(rerank_kernel, dim3(cfg->batch), dim3(RR_THREADS), 0, static_cast<hipStream_t>(stream),
                       C, cfg->n_tree, cfg->topk, cfg->depth, words, cfg->flags, cand_token, cand_score, cand_parent, frontier,
                       cfg->static_tree, root_token, prefix_len,
                       tree_token, tree_parent, tree_depth, tree_cand, position_ids,
                       reinterpret_cast<unsigned long long*>(mask_bits));
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}
