// Host-side runtime around the block calls: the launch trace (per-launch GPU time without an external
// profiler) and the prepared call sequence (a static schedule issued by one call, no interpreter between
// the launches).  No kernels here.
#include <string.h>

#include <mutex>
#include <vector>

#include "../../include/sol_block.h"
#include "launch.h"

namespace sol {

// ---- launch trace --------------------------------------------------------------------------------------
namespace {
struct TracePoint {
    int kind, tag;
    hipEvent_t start, stop;
};
std::mutex g_trace_mutex;
std::vector<TracePoint> g_trace;          // recorded launches, in launch order
std::vector<hipEvent_t> g_trace_pool;     // events created by sol_trace_start, two per launch
size_t g_trace_used = 0;
int g_trace_tag = 0;
}  // namespace

std::atomic<bool> g_trace_on{false};
std::atomic<int> g_trace_kind{0};

bool trace_take_events(hipStream_t, hipEvent_t* start, hipEvent_t* stop) {
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (!g_trace_on.load(std::memory_order_relaxed) || g_trace_used + 2 > g_trace_pool.size()) return false;
    *start = g_trace_pool[g_trace_used++];
    *stop = g_trace_pool[g_trace_used++];
    g_trace.push_back(TracePoint{g_trace_kind.load(std::memory_order_relaxed), g_trace_tag, *start, *stop});
    return true;
}

// ---- prepared sequences ----------------------------------------------------------------------------------
namespace {
struct SeqCall {
    int what;                 // 0 fwd, 1 bwd, 2 loss gradient, 3 max-pool
    sol_block_desc desc;
    const void* a[14];        // pointer arguments in the order of the entry point
    size_t ws_bytes;
    long long numel;
    int i[8];
    int tag;
};
}  // namespace
}  // namespace sol

struct sol_sequence {
    std::vector<sol::SeqCall> calls;
};

using namespace sol;

extern "C" {

SOL_API int sol_trace_start(int32_t capacity) {
    if (capacity < 1 || capacity > (1 << 20)) return SOL_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (g_trace_on.load()) return SOL_ERR_UNSUPPORTED;                 // one trace at a time
    g_trace.clear();
    g_trace.reserve((size_t)capacity);
    g_trace_used = 0;
    while (g_trace_pool.size() < 2 * (size_t)capacity) {
        hipEvent_t ev;
        if (hipEventCreate(&ev) != hipSuccess) {
            (void)hipGetLastError();
            return SOL_ERR_LAUNCH;
        }
        g_trace_pool.push_back(ev);
    }
    g_trace_on.store(true, std::memory_order_release);
    return SOL_OK;
}

SOL_API void sol_trace_tag(int32_t tag) {
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    g_trace_tag = tag;
}

SOL_API int sol_trace_stop(sol_trace_entry* out, int32_t capacity, int32_t* count) {
    if (!count || (capacity > 0 && !out)) return SOL_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (!g_trace_on.load()) return SOL_ERR_UNSUPPORTED;
    g_trace_on.store(false, std::memory_order_release);
    int n = 0;
    int status = SOL_OK;
    for (size_t k = 0; status == SOL_OK && k < g_trace.size(); ++k) {
        float ms = 0.f, since = 0.f;
        if (hipEventSynchronize(g_trace[k].stop) != hipSuccess ||
            hipEventElapsedTime(&ms, g_trace[k].start, g_trace[k].stop) != hipSuccess ||
            hipEventElapsedTime(&since, g_trace[0].start, g_trace[k].start) != hipSuccess) {
            status = SOL_ERR_LAUNCH;
            break;
        }
        if (n < capacity) out[n] = sol_trace_entry{g_trace[k].kind, g_trace[k].tag, ms * 1000.0f, since * 1000.0f};
        ++n;
    }
    if (status != SOL_OK) (void)hipGetLastError();
    *count = n;
    g_trace.clear();
    g_trace_used = 0;
    return status;
}

SOL_API const char* sol_trace_kind_name(int32_t kind) {
    switch (kind) {
        case SOL_TRACE_IGEMM: return "implicit GEMM (pipelined)";
        case SOL_TRACE_IGEMM_GENERAL: return "implicit GEMM (general)";
        case SOL_TRACE_IGEMM_PANEL: return "implicit GEMM (pixel panel in LDS)";
        case SOL_TRACE_IGEMM_REDUCE: return "implicit GEMM (pipelined) + split reduction";
        case SOL_TRACE_IGEMM_PANEL_REDUCE: return "implicit GEMM (pixel panel in LDS) + split reduction";
        case SOL_TRACE_WGRAD: return "weight-gradient GEMM (pipelined)";
        case SOL_TRACE_WGRAD_GENERAL: return "weight-gradient GEMM (general)";
        case SOL_TRACE_WGRAD_REDUCE: return "split reduction";
        case SOL_TRACE_PACK: return "weight re-pack";
        case SOL_TRACE_UNTOUCHED: return "tap-less pixel fill";
        case SOL_TRACE_MASKED_COPY: return "masked copy";
        case SOL_TRACE_SMALLC_PREPARE: return "few-channel prepare";
        case SOL_TRACE_SMALLC_FWD: return "few-channel forward";
        case SOL_TRACE_SMALLC_WGRAD: return "few-channel weight gradient";
        case SOL_TRACE_DIRECT: return "fp32 direct";
        case SOL_TRACE_L1_GRAD: return "L1-loss gradient";
        case SOL_TRACE_MAXPOOL: return "max-pool";
        case SOL_TRACE_OTHER: return "other";
        default: return "unknown";
    }
}

SOL_API sol_sequence* sol_sequence_create(void) { return new (std::nothrow) sol_sequence(); }

SOL_API void sol_sequence_destroy(sol_sequence* seq) { delete seq; }

SOL_API int32_t sol_sequence_length(const sol_sequence* seq) { return seq ? (int32_t)seq->calls.size() : 0; }

SOL_API int sol_sequence_add_fwd(sol_sequence* seq, const sol_block_desc* desc, const void* x, const void* W,
                                 const float* scale, const float* shift, const void* residual, void* y, void* ws,
                                 size_t ws_bytes, int32_t tag) {
    if (!seq || !desc) return SOL_ERR_NULL;
    SeqCall c{};
    c.what = 0;
    c.desc = *desc;
    const void* a[] = {x, W, scale, shift, residual, y, ws};
    memcpy(c.a, a, sizeof a);
    c.ws_bytes = ws_bytes;
    c.tag = tag;
    seq->calls.push_back(c);
    return SOL_OK;
}

SOL_API int sol_sequence_add_bwd(sol_sequence* seq, const sol_block_desc* desc, const void* dy, const void* x, const void* W,
                                 const void* y, void* dx, float* dW, float* dscale, float* dshift, const float* scale,
                                 void* dres, const void* dx_addend, const void* dx_addend_mask, const void* dx_mask,
                                 void* ws, size_t ws_bytes, int32_t tag) {
    if (!seq || !desc) return SOL_ERR_NULL;
    SeqCall c{};
    c.what = 1;
    c.desc = *desc;
    const void* a[] = {dy, x, W, y, dx, dW, dscale, dshift, scale, dres, dx_addend, dx_addend_mask, dx_mask, ws};
    memcpy(c.a, a, sizeof a);
    c.ws_bytes = ws_bytes;
    c.tag = tag;
    seq->calls.push_back(c);
    return SOL_OK;
}

SOL_API int sol_sequence_add_l1_loss_grad(sol_sequence* seq, int32_t dtype, const void* y, const void* t, void* dy,
                                          int64_t numel, int32_t mask_by_y, int32_t tag) {
    if (!seq) return SOL_ERR_NULL;
    SeqCall c{};
    c.what = 2;
    const void* a[] = {y, t, dy};
    memcpy(c.a, a, sizeof a);
    c.numel = numel;
    c.i[0] = dtype;
    c.i[1] = mask_by_y;
    c.tag = tag;
    seq->calls.push_back(c);
    return SOL_OK;
}

SOL_API int sol_sequence_add_maxpool(sol_sequence* seq, int32_t dtype, const void* x, void* y, int32_t N, int32_t H,
                                     int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, int32_t tag) {
    if (!seq) return SOL_ERR_NULL;
    SeqCall c{};
    c.what = 3;
    const void* a[] = {x, y};
    memcpy(c.a, a, sizeof a);
    const int v[] = {dtype, N, H, W, C, k, stride, pad};
    memcpy(c.i, v, sizeof v);
    c.tag = tag;
    seq->calls.push_back(c);
    return SOL_OK;
}

SOL_API int sol_sequence_run(const sol_sequence* seq, int32_t first, int32_t count, void* hip_stream) {
    if (!seq) return SOL_ERR_NULL;
    const int n = (int)seq->calls.size();
    if (first < 0 || count < 0 || first > n || count > n - first) return SOL_ERR_SHAPE;
    const bool tracing = g_trace_on.load(std::memory_order_acquire);
    for (int k = first; k < first + count; ++k) {
        const SeqCall& c = seq->calls[k];
        const void* const* a = c.a;
        if (tracing) sol_trace_tag(c.tag);
        int st;
        switch (c.what) {
            case 0:
                st = sol_block_fwd(&c.desc, a[0], a[1], (const float*)a[2], (const float*)a[3], a[4], (void*)a[5],
                                   (void*)a[6], c.ws_bytes, hip_stream);
                break;
            case 1:
                st = sol_block_bwd(&c.desc, a[0], a[1], a[2], a[3], (void*)a[4], (float*)a[5], (float*)a[6], (float*)a[7],
                                   (const float*)a[8], (void*)a[9], a[10], a[11], a[12], (void*)a[13], c.ws_bytes,
                                   hip_stream);
                break;
            case 2:
                st = sol_l1_loss_grad(c.i[0], a[0], a[1], (void*)a[2], c.numel, c.i[1], hip_stream);
                break;
            default:
                st = sol_maxpool_fwd(c.i[0], a[0], (void*)a[1], c.i[1], c.i[2], c.i[3], c.i[4], c.i[5], c.i[6], c.i[7],
                                     hip_stream);
                break;
        }
        if (st != SOL_OK) return st;
    }
    return SOL_OK;
}

}  // extern "C"
