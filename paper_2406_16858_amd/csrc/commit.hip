// What a round leaves behind for the next one (Section 2.1 of the EAGLE-2 paper: accepted
// draft tokens are kept, the rest of the draft is discarded; Appendix "Implementation
// Details": the KV cache is pre-allocated).
//
//   commit_kv_kernel     copies the keys/values of the accepted path (root first) of every
//                        layer behind the sequence's filled prefix; one launch for all layers
//   commit_kv_fp8_kernel the same for a cache of 8-bit E4M3 codes: rows are divided by the
//                        cache's per-head scale and rounded on their way in
//   commit_round_kernel  emitted tokens, next root, new prefix length, next draft feature
//
// All are plain gathers; 16-byte vector loads and stores, one workgroup per copied row.

#include "common.h"

namespace eagle2 {

constexpr int CM_THREADS = 256;

__global__ __launch_bounds__(CM_THREADS)
void commit_kv_kernel(int N, int D, int row_vec,            // row_vec: 16-byte vectors per (token, all kv heads)
                      long long tree_layer_vec, long long cache_layer_vec,
                      const int* __restrict__ accept_len, const int* __restrict__ accept_path,
                      const long long* __restrict__ kv_offsets, const int* __restrict__ prefix_len,
                      const u32x4* __restrict__ K_tree, const u32x4* __restrict__ V_tree,
                      u32x4* __restrict__ K_cache, u32x4* __restrict__ V_cache) {
    const int i = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
    int len = accept_len[b];
    if (len < 0) return;                                     // acceptance reported a failure: nothing is committed
    len = len > D ? D : len;
    if (i > len) return;
    const int row = accept_path[(size_t)b * (D + 1) + i];
    const int P = prefix_len[b];
    if (row < 0 || row >= N || P < 0) return;
    const long long dst = kv_offsets[b] + P + i;
    if (dst >= kv_offsets[b + 1]) return;                    // beyond the sequence's region: dropped
    const size_t src_v = (size_t)layer * tree_layer_vec + ((size_t)b * N + row) * row_vec;
    const size_t dst_v = (size_t)layer * cache_layer_vec + (size_t)dst * row_vec;
    for (int v = threadIdx.x; v < row_vec; v += CM_THREADS) {
        const u32x4 kk = K_tree[src_v + v], vv = V_tree[src_v + v];
        K_cache[dst_v + v] = kk;
        V_cache[dst_v + v] = vv;
    }
}

// sixteen bf16 values -> sixteen E4M3 codes of x / scale: correctly rounded float32 quotient, clamped
// to the largest finite code (448), rounded to nearest even by the conversion instruction
__device__ __forceinline__ u32x4 quantize16(const u32x4& a, const u32x4& b, float scale) {
    u32x4 out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const unsigned w0 = j < 2 ? a[2 * j] : b[2 * j - 4], w1 = j < 2 ? a[2 * j + 1] : b[2 * j - 3];
        float q[4] = {__uint_as_float(w0 << 16), __uint_as_float(w0 & 0xffff0000u),
                      __uint_as_float(w1 << 16), __uint_as_float(w1 & 0xffff0000u)};
#pragma unroll
        for (int e = 0; e < 4; ++e) q[e] = fminf(fmaxf(__fdiv_rn(q[e], scale), -448.f), 448.f);
        int r = __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], 0, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], r, true);
        out[j] = (unsigned)r;
    }
    return out;
}

// row_vec8: 16-byte vectors of codes per (token, all kv heads); vec_per_head = dh / 16
__global__ __launch_bounds__(CM_THREADS)
void commit_kv_fp8_kernel(int N, int D, int row_vec8, int vec_per_head, int Hkv,
                          long long tree_layer_vec, long long cache_layer_vec,
                          const int* __restrict__ accept_len, const int* __restrict__ accept_path,
                          const long long* __restrict__ kv_offsets, const int* __restrict__ prefix_len,
                          const u32x4* __restrict__ K_tree, const u32x4* __restrict__ V_tree,
                          u32x4* __restrict__ K_cache, u32x4* __restrict__ V_cache,
                          const float* __restrict__ k_scale, const float* __restrict__ v_scale) {
    const int i = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
    int len = accept_len[b];
    if (len < 0) return;                                     // acceptance reported a failure: nothing is committed
    len = len > D ? D : len;
    if (i > len) return;
    const int row = accept_path[(size_t)b * (D + 1) + i];
    const int P = prefix_len[b];
    if (row < 0 || row >= N || P < 0) return;
    const long long dst = kv_offsets[b] + P + i;
    if (dst >= kv_offsets[b + 1]) return;                    // beyond the sequence's region: dropped
    const size_t src_v = (size_t)layer * tree_layer_vec + ((size_t)b * N + row) * (2 * (size_t)row_vec8);
    const size_t dst_v = (size_t)layer * cache_layer_vec + (size_t)dst * row_vec8;
    for (int v = threadIdx.x; v < row_vec8; v += CM_THREADS) {
        const int h = v / vec_per_head;
        const float ks = k_scale[(size_t)layer * Hkv + h], vs = v_scale[(size_t)layer * Hkv + h];
        K_cache[dst_v + v] = quantize16(K_tree[src_v + 2 * v], K_tree[src_v + 2 * v + 1], ks);
        V_cache[dst_v + v] = quantize16(V_tree[src_v + 2 * v], V_tree[src_v + 2 * v + 1], vs);
    }
}

__global__ __launch_bounds__(CM_THREADS)
void commit_round_kernel(int N, int D, int hid_vec,
                         const int* __restrict__ accept_len, const int* __restrict__ accept_path,
                         const int* __restrict__ tree_token, const int* __restrict__ bonus_token,
                         const u32x4* __restrict__ target_hidden,
                         int* __restrict__ out_tokens, int* __restrict__ root_token, int* __restrict__ prefix_len,
                         u32x4* __restrict__ next_hidden) {
    const int b = blockIdx.x, tid = threadIdx.x;
    int len = accept_len[b];
    if (len < 0) {
        // acceptance reported a failure for this sequence: no token is emitted and the root, the prefix
        // length and the next feature stay as they were, so the caller can run the round again
        if (tid <= D) out_tokens[(size_t)b * (D + 1) + tid] = -1;
        return;
    }
    len = len > D ? D : len;
    const int* path = accept_path + (size_t)b * (D + 1);
    const int bonus = bonus_token[b];
    if (tid <= D) {
        int t = -1;
        if (tid < len) {
            const int row = path[tid + 1];
            t = (row >= 0 && row < N) ? tree_token[(size_t)b * N + row] : -1;
        } else if (tid == len) {
            t = bonus;
        }
        out_tokens[(size_t)b * (D + 1) + tid] = t;
    }
    if (tid == 0) {
        root_token[b] = bonus;
        prefix_len[b] += len + 1;
    }
    if (next_hidden != nullptr) {
        int row = path[len];
        if (row < 0 || row >= N) row = 0;
        const u32x4* src = target_hidden + ((size_t)b * N + row) * hid_vec;
        for (int v = tid; v < hid_vec; v += CM_THREADS) next_hidden[(size_t)b * hid_vec + v] = src[v];
    }
}

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_commit_kv(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int32_t n_layers,
                                const int32_t* accept_len, const int32_t* accept_path,
                                const int64_t* kv_offsets, const int32_t* prefix_len,
                                const void* K_tree, const void* V_tree, int64_t tree_layer_stride,
                                void* K_cache, void* V_cache, int64_t cache_layer_stride, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    rc = validate_attn(cfg, attn);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(accept_len && accept_path && kv_offsets && prefix_len && K_tree && V_tree && K_cache && V_cache,
               EAGLE2_ERR_ARG, "eagle2_commit_kv: null pointer argument");
    E2_REQUIRE(n_layers >= 1 && n_layers <= 65535, EAGLE2_ERR_ARG, "eagle2_commit_kv: n_layers %d outside [1, 65535]", n_layers);
    E2_REQUIRE(cfg->batch <= 65535, EAGLE2_ERR_SHAPE, "eagle2_commit_kv: batch %d exceeds 65535", cfg->batch);
    E2_REQUIRE(aligned16(K_tree) && aligned16(V_tree) && aligned16(K_cache) && aligned16(V_cache), EAGLE2_ERR_ARG,
               "eagle2_commit_kv: tensors must be 16-byte aligned");
    const int64_t row_bytes = (int64_t)attn->n_kv_heads * attn->head_dim * elem_size(cfg);     // a multiple of 128
    const int64_t es = elem_size(cfg);
    E2_REQUIRE(tree_layer_stride >= 0 && cache_layer_stride >= 0 && (tree_layer_stride * es) % 16 == 0 &&
               (cache_layer_stride * es) % 16 == 0, EAGLE2_ERR_ARG,
               "eagle2_commit_kv: layer strides must be non-negative multiples of 16 bytes");
    if (n_layers > 1)
        E2_REQUIRE(tree_layer_stride * es >= (int64_t)cfg->batch * cfg->n_tree * row_bytes &&
                   cache_layer_stride * es >= attn->total_prefix * row_bytes, EAGLE2_ERR_ARG,
                   "eagle2_commit_kv: layer strides smaller than one layer");
    dim3 grid(cfg->depth + 1, cfg->batch, n_layers);
    hipLaunchKernelGGL(commit_kv_kernel, grid, dim3(CM_THREADS), 0, static_cast<hipStream_t>(stream),
                       cfg->n_tree, cfg->depth, (int)(row_bytes / 16), (long long)(tree_layer_stride * es / 16),
                       (long long)(cache_layer_stride * es / 16), accept_len, accept_path,
                       reinterpret_cast<const long long*>(kv_offsets), prefix_len,
                       static_cast<const u32x4*>(K_tree), static_cast<const u32x4*>(V_tree),
                       static_cast<u32x4*>(K_cache), static_cast<u32x4*>(V_cache));
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

extern "C" int eagle2_commit_kv_fp8(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int32_t n_layers,
                                    const int32_t* accept_len, const int32_t* accept_path,
                                    const int64_t* kv_offsets, const int32_t* prefix_len,
                                    const void* K_tree, const void* V_tree, int64_t tree_layer_stride,
                                    void* K_cache8, void* V_cache8, int64_t cache_layer_stride,
                                    const float* k_scale, const float* v_scale, void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    rc = validate_attn(cfg, attn);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(cfg->dtype == EAGLE2_DTYPE_BF16, EAGLE2_ERR_SHAPE, "eagle2_commit_kv_fp8: the 8-bit cache goes with dtype bf16 only");
    E2_REQUIRE(accept_len && accept_path && kv_offsets && prefix_len && K_tree && V_tree && K_cache8 && V_cache8 && k_scale && v_scale,
               EAGLE2_ERR_ARG, "eagle2_commit_kv_fp8: null pointer argument");
    E2_REQUIRE(n_layers >= 1 && n_layers <= 65535, EAGLE2_ERR_ARG, "eagle2_commit_kv_fp8: n_layers %d outside [1, 65535]", n_layers);
    E2_REQUIRE(cfg->batch <= 65535, EAGLE2_ERR_SHAPE, "eagle2_commit_kv_fp8: batch %d exceeds 65535", cfg->batch);
    E2_REQUIRE(aligned16(K_tree) && aligned16(V_tree) && aligned16(K_cache8) && aligned16(V_cache8), EAGLE2_ERR_ARG,
               "eagle2_commit_kv_fp8: tensors must be 16-byte aligned");
    const int64_t row_codes = (int64_t)attn->n_kv_heads * attn->head_dim;                       // a multiple of 64
    E2_REQUIRE(tree_layer_stride >= 0 && cache_layer_stride >= 0 && (tree_layer_stride * 2) % 16 == 0 &&
               cache_layer_stride % 16 == 0, EAGLE2_ERR_ARG,
               "eagle2_commit_kv_fp8: layer strides must be non-negative multiples of 16 bytes");
    if (n_layers > 1)
        E2_REQUIRE(tree_layer_stride >= (int64_t)cfg->batch * cfg->n_tree * row_codes &&
                   cache_layer_stride >= attn->total_prefix * row_codes, EAGLE2_ERR_ARG,
                   "eagle2_commit_kv_fp8: layer strides smaller than one layer");
    dim3 grid(cfg->depth + 1, cfg->batch, n_layers);
    hipLaunchKernelGGL(commit_kv_fp8_kernel, grid, dim3(CM_THREADS), 0, static_cast<hipStream_t>(stream),
                       cfg->n_tree, cfg->depth, (int)(row_codes / 16), attn->head_dim / 16, attn->n_kv_heads,
                       (long long)(tree_layer_stride * 2 / 16), (long long)(cache_layer_stride / 16), accept_len, accept_path,
                       reinterpret_cast<const long long*>(kv_offsets), prefix_len,
                       static_cast<const u32x4*>(K_tree), static_cast<const u32x4*>(V_tree),
                       static_cast<u32x4*>(K_cache8), static_cast<u32x4*>(V_cache8), k_scale, v_scale);
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}

extern "C" int eagle2_commit_round(const eagle2_cfg* cfg, const int32_t* accept_len, const int32_t* accept_path,
                                   const int32_t* tree_token, const int32_t* bonus_token, const void* target_hidden,
                                   int32_t* out_tokens, int32_t* root_token, int32_t* prefix_len, void* next_hidden,
                                   void* stream) {
    int rc = validate_cfg(cfg);
    if (rc != EAGLE2_OK) return rc;
    E2_REQUIRE(accept_len && accept_path && tree_token && bonus_token && out_tokens && root_token && prefix_len,
               EAGLE2_ERR_ARG, "eagle2_commit_round: null pointer argument");
    E2_REQUIRE((target_hidden == nullptr) == (next_hidden == nullptr), EAGLE2_ERR_ARG,
               "eagle2_commit_round: target_hidden and next_hidden must be given together");
    E2_REQUIRE(aligned16(target_hidden) && aligned16(next_hidden), EAGLE2_ERR_ARG,
               "eagle2_commit_round: tensors must be 16-byte aligned");
    E2_REQUIRE(cfg->depth + 1 <= CM_THREADS, EAGLE2_ERR_SHAPE, "eagle2_commit_round: depth too large");
    const int hid_vec = (int)((int64_t)cfg->hidden * elem_size(cfg) / 16);                    // hidden rows are multiples of 1 KiB
    hipLaunchKernelGGL(commit_round_kernel, dim3(cfg->batch), dim3(CM_THREADS), 0, static_cast<hipStream_t>(stream),
                       cfg->n_tree, cfg->depth, hid_vec, accept_len, accept_path, tree_token, bonus_token,
                       static_cast<const u32x4*>(target_hidden), out_tokens, root_token, prefix_len,
                       static_cast<u32x4*>(next_hidden));
    E2_HIP(hipGetLastError());
    return EAGLE2_OK;
}
