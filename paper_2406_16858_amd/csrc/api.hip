// Library-wide pieces: version, error text, shape validation, workspace sizing and the
// optional kernel-timing hooks used by the benchmark.
#include "common.h"
#include <stdarg.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <vector>

namespace eagle2 {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int validate_cfg(const eagle2_cfg* c) {
    E2_REQUIRE(c != nullptr, EAGLE2_ERR_ARG, "cfg is null");
    E2_REQUIRE(c->dtype == EAGLE2_DTYPE_F32 || c->dtype == EAGLE2_DTYPE_BF16, EAGLE2_ERR_SHAPE,
               "dtype %d is neither float32 nor bfloat16", c->dtype);
    E2_REQUIRE(c->batch >= 1 && c->batch <= 4096, EAGLE2_ERR_SHAPE, "batch %d outside [1, 4096]", c->batch);
    E2_REQUIRE(c->topk >= 1 && c->topk <= EAGLE2_MAX_TOPK, EAGLE2_ERR_SHAPE, "topk %d outside [1, %d]", c->topk, EAGLE2_MAX_TOPK);
    E2_REQUIRE(c->vocab >= 16 && c->vocab >= c->topk, EAGLE2_ERR_SHAPE, "vocab %d smaller than 16 or than topk", c->vocab);
    E2_REQUIRE(c->depth >= 1 && c->depth <= 64, EAGLE2_ERR_SHAPE, "depth %d outside [1, 64]", c->depth);
    E2_REQUIRE(c->hidden >= 1 && ((int64_t)c->hidden * elem_size(c)) % 1024 == 0, EAGLE2_ERR_SHAPE,
               "hidden %d: a row of W must be a multiple of 1024 bytes", c->hidden);
    const int64_t C = (int64_t)c->topk + (int64_t)(c->depth - 1) * c->topk * c->topk;
    E2_REQUIRE(C <= EAGLE2_MAX_CAND, EAGLE2_ERR_SHAPE, "%lld candidates per round exceed %d", (long long)C, EAGLE2_MAX_CAND);
    E2_REQUIRE(c->n_tree >= 2 && c->n_tree <= EAGLE2_MAX_TREE && c->n_tree - 1 <= C, EAGLE2_ERR_SHAPE,
               "n_tree %d outside [2, min(%d, C+1 = %lld)]", c->n_tree, EAGLE2_MAX_TREE, (long long)C + 1);
    E2_REQUIRE((c->flags & ~(EAGLE2_FLAG_RANK_BY_CONFIDENCE | EAGLE2_FLAG_NO_RERANK | EAGLE2_FLAG_STATIC_TREE)) == 0, EAGLE2_ERR_ARG,
               "flags 0x%x contain unknown bits", c->flags);
    if (c->flags & EAGLE2_FLAG_STATIC_TREE) {
        E2_REQUIRE(c->flags == EAGLE2_FLAG_STATIC_TREE, EAGLE2_ERR_ARG, "EAGLE2_FLAG_STATIC_TREE excludes the other flags");
        E2_REQUIRE(c->static_tree != nullptr, EAGLE2_ERR_ARG, "EAGLE2_FLAG_STATIC_TREE needs cfg->static_tree");
    }
    if (c->flags & EAGLE2_FLAG_NO_RERANK)
        E2_REQUIRE(c->n_tree == c->depth * c->topk + 1, EAGLE2_ERR_SHAPE,
                   "without reranking the tree has depth*topk + 1 = %d rows, n_tree is %d", c->depth * c->topk + 1, c->n_tree);
    E2_REQUIRE((int64_t)c->vocab * c->n_tree * (int64_t)c->batch < (1ll << 40), EAGLE2_ERR_SHAPE, "logit tensor too large");
    return EAGLE2_OK;
}

int validate_attn(const eagle2_cfg* c, const eagle2_attn_cfg* a) {
    E2_REQUIRE(a != nullptr, EAGLE2_ERR_ARG, "attn cfg is null");
    E2_REQUIRE(a->head_dim == 64 || a->head_dim == 128, EAGLE2_ERR_SHAPE, "head_dim %d is not 64 or 128", a->head_dim);
    E2_REQUIRE(a->n_kv_heads >= 1 && a->n_q_heads >= a->n_kv_heads && a->n_q_heads % a->n_kv_heads == 0 &&
               a->n_q_heads <= 1024, EAGLE2_ERR_SHAPE, "heads %d/%d: q heads must be a multiple of kv heads", a->n_q_heads, a->n_kv_heads);
    E2_REQUIRE(a->total_prefix >= 0 && a->total_prefix < (1ll << 31), EAGLE2_ERR_SHAPE, "total_prefix %lld out of range", (long long)a->total_prefix);
    E2_REQUIRE(a->scale >= 0.f, EAGLE2_ERR_ARG, "negative attention scale");
    (void)c;
    return EAGLE2_OK;
}

int device_cu_count() {
    static int cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

// ---- kernel timing ---------------------------------------------------------------
// The only mutable global state of the library.  Events are created when timing is switched on
// (a fixed pool per slot), never inside an entry point of the method; a launch that finds the pool
// exhausted is simply not timed.
constexpr size_t TIMING_POOL = 4096;               // events per slot = 2048 timed launches between two reads
struct TimingSlot { std::vector<hipEvent_t> ev; size_t used = 0; };
static std::mutex g_tmu;
static std::atomic<bool> g_timing{false};
static TimingSlot g_slots[2];

void timing_begin(int which, hipStream_t st) {
    if (!g_timing.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lk(g_tmu);
    TimingSlot& s = g_slots[which];
    if ((s.used & 1) != 0 || s.used + 2 > s.ev.size()) return;  // unmatched begin, or no room left for a pair
    (void)hipEventRecord(s.ev[s.used++], st);
}
void timing_end(int which, hipStream_t st) {
    if (!g_timing.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lk(g_tmu);
    TimingSlot& s = g_slots[which];
    if ((s.used & 1) == 0 || s.used >= s.ev.size()) return;    // no begin was recorded for this launch
    (void)hipEventRecord(s.ev[s.used++], st);
}

}  // namespace eagle2

using namespace eagle2;

extern "C" int eagle2_version(void) { return 100; }

extern "C" const char* eagle2_last_error(void) { return g_err; }

extern "C" size_t eagle2_workspace_bytes(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn) {
    if (validate_cfg(cfg) != EAGLE2_OK) return 0;
    size_t n = expand_workspace(cfg);
    size_t m = rerank_workspace(cfg);
    if (m > n) n = m;
    m = accept_workspace(cfg);
    if (m > n) n = m;
    if (attn != nullptr) {
        if (validate_attn(cfg, attn) != EAGLE2_OK) return 0;
        m = attn_workspace(cfg, attn);
        if (m > n) n = m;
    }
    return n;
}

extern "C" int eagle2_kernel_timing_enable(int32_t enable) {
    std::lock_guard<std::mutex> lk(g_tmu);
    if (enable) {
        for (auto& s : g_slots) {
            while (s.ev.size() < TIMING_POOL) {
                hipEvent_t e;
                E2_HIP(hipEventCreate(&e));
                s.ev.push_back(e);
            }
        }
    }
    for (auto& s : g_slots) s.used = 0;
    g_timing.store(enable != 0, std::memory_order_release);
    return EAGLE2_OK;
}

extern "C" int eagle2_kernel_timing_read(int32_t which, double* total_ms, int32_t* launches) {
    E2_REQUIRE(which == 0 || which == 1, EAGLE2_ERR_ARG, "timing slot %d does not exist", which);
    E2_REQUIRE(total_ms && launches, EAGLE2_ERR_ARG, "null output pointer");
    std::lock_guard<std::mutex> lk(g_tmu);
    TimingSlot& s = g_slots[which];
    double tot = 0.0;
    int n = 0;
    for (size_t i = 0; i + 1 < s.used; i += 2) {
        E2_HIP(hipEventSynchronize(s.ev[i + 1]));
        float ms = 0.f;
        E2_HIP(hipEventElapsedTime(&ms, s.ev[i], s.ev[i + 1]));
        tot += ms;
        ++n;
    }
    s.used = 0;
    *total_ms = tot;
    *launches = n;
    return EAGLE2_OK;
}
