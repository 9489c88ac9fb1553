// Host-callable launchers of the kernels (one translation unit per kernel family).
#pragma once

#include "common.h"

#include <hip/hip_ext.h>

#include <atomic>

namespace sol {

// Kernels that need more than 64 KiB of dynamic LDS must have their limit raised; that is a driver
// call, so it is made once per kernel instantiation (per process: one process drives one GPU) instead
// of once per launch.  `granted` is the instantiation's own counter.
inline hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes, std::atomic<size_t>& granted) {
    if (granted.load(std::memory_order_acquire) >= bytes) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) granted.store(bytes, std::memory_order_release);
    return e;
}

// Launch trace: while a trace is on (sol_trace_start), every kernel launch of the library carries a start and a
// stop event of its own (the runtime stamps them from the dispatch itself, so the time between them is the
// kernel's execution time, as a profiler would report it, without a barrier between kernels).  trace_point names
// the kind of the launches that follow; off, a launch pays one relaxed atomic load.
extern std::atomic<bool> g_trace_on;
extern std::atomic<int> g_trace_kind;
bool trace_take_events(hipStream_t stream, hipEvent_t* start, hipEvent_t* stop);
inline void trace_point(hipStream_t, int kind) {
    if (g_trace_on.load(std::memory_order_relaxed)) g_trace_kind.store(kind, std::memory_order_relaxed);
}
#define SOL_LAUNCH(kern, grid, block, smem, stream, ...)                                                           \
    do {                                                                                                           \
        hipEvent_t sol_ev0_, sol_ev1_;                                                                             \
        if (sol::g_trace_on.load(std::memory_order_relaxed) && sol::trace_take_events(stream, &sol_ev0_, &sol_ev1_)) \
            hipExtLaunchKernelGGL(kern, grid, block, smem, stream, sol_ev0_, sol_ev1_, 0, __VA_ARGS__);            \
        else                                                                                                       \
            hipLaunchKernelGGL(kern, grid, block, smem, stream, __VA_ARGS__);                                      \
    } while (0)

struct DirectParams {
    const float* x;
    const float* W;
    const float* scale;
    const float* shift;
    const float* res;
    float* y;
    const float* dy;
    const float* ymask;       // y of the block when it has a ReLU, else null
    float* dx;
    const float* addend;
    const float* addend_mask;
    const float* dx_mask;
    float* G;                 // unscaled weight gradient [C_out][K] (one split)
    float* dshift_partial;    // [C_out]
    int N, H, W_, C_in, C_out, KH, KW, stride, pad, Ho, Wo, relu;
};


struct SmallCParams {          // convolution with at most 4 input channels, 64 output channels, stride 2
    const bf16_t* x;           // [N][H][W][C_in]
    bf16_t* xp;                // workspace: [N][H][W][4], channel-padded copy of x
    const bf16_t* Wt;          // [64][KH][KW][C_in]
    bf16_t* wp;                // workspace: weights as MFMA operand image, [2*KH][64][2][8]
    const float* scale;
    const float* shift;
    bf16_t* y;                 // [N][Ho][Wo][64]
    int N, H, W, C_in, KH, KW, pad, Ho, Wo, relu;
};
struct SmallCWgradParams {     // weight gradient of the same layers (dy already masked)
    const bf16_t* dy;          // [N][Ho][Wo][64]
    const bf16_t* xp;          // channel-padded image (smallc_prepare)
    const bf16_t* Wt;          // for dscale
    const float* scale;
    float* partial;            // workspace: [nparts][64][264] fp32
    float* dW;                 // [64][KH][KW][C_in]
    float* dscale;
    float* dshift;
    int N, H, W, C_in, KH, KW, pad, Ho, Wo, nparts, accumulate;
};
bool smallc_wgrad_supported(int C_in, int C_out, int KH, int KW, int stride);
int smallc_wgrad_parts(int N, int Ho, int Wo);
size_t smallc_wgrad_partial_bytes(int nparts);
hipError_t launch_smallc_wgrad(const SmallCWgradParams& p, hipStream_t stream);
bool smallc_fwd_supported(int C_in, int C_out, int KH, int KW, int stride);
size_t smallc_padded_image_bytes(int N, int H, int W);
size_t smallc_packed_weight_bytes(int KH);
hipError_t launch_smallc_prepare(const SmallCParams& p, hipStream_t stream);
hipError_t launch_smallc_fwd(const SmallCParams& p, hipStream_t stream);

hipError_t launch_igemm(const IgemmParams& p, int tile, bool vec, bool mask, hipStream_t stream);
void igemm_tile_shape(int tile, int* bp, int* bc);
hipError_t launch_igemm_fast(const IgemmParams& p, int tile, int stages, hipStream_t stream);
void igemm_fast_tile_shape(int tile, int* bp, int* bc);
bool igemm_panel_eligible(const IgemmParams& p);
int plan_igemm_panel(IgemmParams& p, int tiles_per_workgroup);
hipError_t launch_igemm_panel(const IgemmParams& p, hipStream_t stream);
hipError_t launch_wgrad(const WgradParams& p, bool vec, bool mask, hipStream_t stream);
hipError_t launch_wgrad_fast(const WgradParams& p, int stages, hipStream_t stream);
hipError_t launch_wgrad_reduce(const ReduceParams& p, hipStream_t stream);
hipError_t launch_direct_fwd_f32(const DirectParams& p, hipStream_t s);
hipError_t launch_direct_dgrad_f32(const DirectParams& p, hipStream_t s);
hipError_t launch_direct_wgrad_f32(const DirectParams& p, hipStream_t s);
hipError_t launch_pack_dgrad_weights(const PackParams& p, hipStream_t s);
hipError_t launch_untouched_pixels(void* dx, const void* addend, const void* addend_mask, const void* out_mask, int N,
                                   int H, int W, int C, int KH, int KW, int stride, int pad, hipStream_t s);
hipError_t launch_masked_copy(int dtype, const void* dy, const void* y, void* dres, long long numel, hipStream_t s);
hipError_t launch_l1_grad(int dtype, const void* y, const void* t, void* dy, long long numel, int mask_by_y,
                          hipStream_t s);
hipError_t launch_maxpool(int dtype, const void* x, void* y, int N, int H, int W, int C, int k, int stride, int pad,
                          hipStream_t s);

}  // namespace sol
