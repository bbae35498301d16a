// Internal helpers shared by the translation units of libeagle2_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <limits.h>
#include "../../include/eagle2.h"

namespace eagle2 {

// ---- host-side error reporting -------------------------------------------------
void set_error(const char* fmt, ...);
int  validate_cfg(const eagle2_cfg* cfg);          // EAGLE2_OK or an error code (message set)
int  validate_attn(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn);

#define E2_REQUIRE(cond, code, ...)                         \
    do { if (!(cond)) { ::eagle2::set_error(__VA_ARGS__); return (code); } } while (0)

#define E2_HIP(call)                                                            \
    do { hipError_t e_ = (call);                                                \
         if (e_ != hipSuccess) {                                                \
             ::eagle2::set_error("%s failed: %s", #call, hipGetErrorString(e_)); \
             return EAGLE2_ERR_HIP; } } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static inline int n_cand(const eagle2_cfg* c) { return c->topk + (c->depth - 1) * c->topk * c->topk; }
static inline int n_draft_rows(const eagle2_cfg* c) { return 1 + (c->depth - 1) * c->topk; }
static inline int elem_size(const eagle2_cfg* c) { return c->dtype == EAGLE2_DTYPE_F32 ? 4 : 2; }

// per-entry-point workspace needs (bytes)
size_t expand_workspace(const eagle2_cfg* cfg);
size_t rerank_workspace(const eagle2_cfg* cfg);
size_t attn_workspace(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn);
size_t attn_workspace_rows(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int nq);   // nq query rows only
size_t accept_workspace(const eagle2_cfg* cfg);

int device_cu_count();

// dense float32 out[M, N] = X[M, K] . W[N, K]^T for more than 16 rows, W streamed once per 160 rows
// (X row (b, s) at X + b * x_seq_bytes + s * row_bytes; hp_ws: ceil(M/16)*16 * row_bytes bytes of scratch;
// done_count[0 .. n_done) is zeroed as a side job, n_done may be 0)
int gemm_rows(bool bf16, const void* X, int64_t x_seq_bytes, int M, int F, const void* W, int N, int row_bytes,
              float* out, void* hp_ws, unsigned* done_count, int n_done, hipStream_t st);

// tree attention restricted to the query rows q0 .. q0+nq-1 (same arguments as eagle2_tree_attn otherwise;
// k_scale/v_scale non-null: the prefix keys/values are 8-bit E4M3 codes with these per-KV-head scales)
int tree_attn_rows(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int q0, int nq,
                   const void* Q, const void* K_prefix, const void* V_prefix, const float* k_scale, const float* v_scale,
                   const int64_t* kv_offsets, const int32_t* kv_len,
                   const void* K_tree, const void* V_tree, const uint64_t* mask_bits, void* O, float* lse,
                   void* workspace, size_t workspace_bytes, void* stream);

// ---- optional kernel timing ----------------------------------------------------
// record_begin/end are no-ops unless timing is enabled.
void timing_begin(int which, hipStream_t s);
void timing_end(int which, hipStream_t s);

// ---- device helpers --------------------------------------------------------------
#ifdef __HIPCC__
typedef float    floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4   __attribute__((ext_vector_type(4)));
typedef unsigned u32x2   __attribute__((ext_vector_type(2)));
typedef float    float2v __attribute__((ext_vector_type(2)));
typedef __bf16   bf16x8  __attribute__((ext_vector_type(8)));

// ---- wave-wide reductions on the DPP data path -------------------------------------------
// Four symmetric exchanges inside each row of 16 lanes (lane^1, lane^2, mirror within 8,
// mirror within 16) leave every lane of a row with the row's result; the four row results
// are then read with v_readlane and combined in a fixed order.  No LDS traffic, unlike
// __shfl_xor.  All callers run with full waves in wave-uniform control flow.
constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;
constexpr int DPP_MIRROR = 0x140;

template <int CTRL> __device__ __forceinline__ int dpp_mov(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL> __device__ __forceinline__ double dpp_mov(double v) {
    const int lo = dpp_mov<CTRL>(__double2loint(v)), hi = dpp_mov<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}
// The value of lane^16 / lane^32, on the vector ALU (gfx950's row and half-wave swaps) instead of the
// LDS crossbar a shuffle uses.  permlane16_swap(x, x) returns (rows 0,0,2,2 ; rows 1,1,3,3) of x, so an
// even row finds its neighbour in the second result and an odd row in the first; permlane32_swap(x, x)
// returns (lower half twice ; upper half twice).
__device__ __forceinline__ int lane_xor16(int v) {
    const u32x2 r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((threadIdx.x & 16) ? r[0] : r[1]);
}
__device__ __forceinline__ int lane_xor32(int v) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float lane_xor16(float v) { return __int_as_float(lane_xor16(__float_as_int(v))); }
__device__ __forceinline__ float lane_xor32(float v) { return __int_as_float(lane_xor32(__float_as_int(v))); }
__device__ __forceinline__ int read_lane(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
// lane index held in a register (must be wave-uniform)
__device__ __forceinline__ int read_lane_dyn(int v, int l) { return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(l)); }
__device__ __forceinline__ float read_lane_dyn(float v, int l) { return __int_as_float(read_lane_dyn(__float_as_int(v), l)); }
__device__ __forceinline__ double read_lane_dyn(double v, int l) {
    return __hiloint2double(read_lane_dyn(__double2hiint(v), l), read_lane_dyn(__double2loint(v), l));
}
__device__ __forceinline__ float read_lane(float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); }
__device__ __forceinline__ double read_lane(double v, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l), __builtin_amdgcn_readlane(__double2loint(v), l));
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_mov<DPP_XOR1>(v));
    v = fmaxf(v, dpp_mov<DPP_XOR2>(v));
    v = fmaxf(v, dpp_mov<DPP_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_mov<DPP_MIRROR>(v));
    return fmaxf(fmaxf(read_lane(v, 0), read_lane(v, 16)), fmaxf(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ double wave_maxd(double v) {
    v = fmax(v, dpp_mov<DPP_XOR1>(v));
    v = fmax(v, dpp_mov<DPP_XOR2>(v));
    v = fmax(v, dpp_mov<DPP_HALF_MIRROR>(v));
    v = fmax(v, dpp_mov<DPP_MIRROR>(v));
    return fmax(fmax(read_lane(v, 0), read_lane(v, 16)), fmax(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ float wave_sumf(float v) {
    v += dpp_mov<DPP_XOR1>(v);
    v += dpp_mov<DPP_XOR2>(v);
    v += dpp_mov<DPP_HALF_MIRROR>(v);
    v += dpp_mov<DPP_MIRROR>(v);
    return ((read_lane(v, 0) + read_lane(v, 16)) + read_lane(v, 32)) + read_lane(v, 48);
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_mov<DPP_XOR1>(v);
    v += dpp_mov<DPP_XOR2>(v);
    v += dpp_mov<DPP_HALF_MIRROR>(v);
    v += dpp_mov<DPP_MIRROR>(v);
    return ((read_lane(v, 0) + read_lane(v, 16)) + read_lane(v, 32)) + read_lane(v, 48);
}
// The wave waits until all of its outstanding vector-memory loads and stores have completed
// (s_waitcnt vmcnt(0); the export and LDS/scalar counters are left at their maxima).  Used before a
// device-scope counter increment that publishes earlier device-scope stores of the same wave.
__device__ __forceinline__ void wait_vector_memory() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// candidate order: higher value first, then lower index
// (bitwise operators on purpose: the short-circuit forms compile to divergent branches around two of
// the three comparisons)
__device__ __forceinline__ bool ranks_before(float va, int ia, float vb, int ib) {
    return (va > vb) | ((va == vb) & (ia < ib));
}
__device__ __forceinline__ bool ranks_before(double va, int ia, double vb, int ib) {
    return (va > vb) | ((va == vb) & (ia < ib));
}
// every lane ends with the wave's best (value, index) and the payload that travels with it
template <typename T>
__device__ __forceinline__ void wave_best(T& v, int& i, int& pay) {
#define E2_BEST_STEP(CTRL)                                                                     \
    {                                                                                          \
        const T ov = dpp_mov<CTRL>(v);                                                         \
        const int oi = dpp_mov<CTRL>(i), op = dpp_mov<CTRL>(pay);                              \
        if (ranks_before(ov, oi, v, i)) { v = ov; i = oi; pay = op; }                          \
    }
    E2_BEST_STEP(DPP_XOR1) E2_BEST_STEP(DPP_XOR2) E2_BEST_STEP(DPP_HALF_MIRROR) E2_BEST_STEP(DPP_MIRROR)
#undef E2_BEST_STEP
    T bv = read_lane(v, 0);
    int bi = read_lane(i, 0), bp = read_lane(pay, 0);
#pragma unroll
    for (int r = 1; r < 4; ++r) {
        const T rv = read_lane(v, 16 * r);
        const int ri = read_lane(i, 16 * r), rp = read_lane(pay, 16 * r);
        if (ranks_before(rv, ri, bv, bi)) { bv = rv; bi = ri; bp = rp; }
    }
    v = bv; i = bi; pay = bp;
}
template <typename T>
__device__ __forceinline__ void wave_best(T& v, int& i) { int pay = 0; wave_best(v, i, pay); }
#endif

}  // namespace eagle2
