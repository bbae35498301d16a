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
size_t accept_workspace(const eagle2_cfg* cfg);

int device_cu_count();

// ---- optional kernel timing ----------------------------------------------------
// record_begin/end are no-ops unless timing is enabled.
void timing_begin(int which, hipStream_t s);
void timing_end(int which, hipStream_t s);

// ---- device helpers --------------------------------------------------------------
#ifdef __HIPCC__
typedef float    floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4   __attribute__((ext_vector_type(4)));
typedef unsigned u32x2   __attribute__((ext_vector_type(2)));
typedef __bf16   bf16x8  __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_maxd(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}
// candidate order: higher value first, then lower index
__device__ __forceinline__ bool ranks_before(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}
__device__ __forceinline__ bool ranks_before(double va, int ia, double vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}
#endif

}  // namespace eagle2
