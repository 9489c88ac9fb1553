/*
 * sol_block.h -- C-ABI of the fused layer block
 *
 *      y = [ReLU]( scale[c] * conv(x, W)[.., c] + shift[c] [+ residual] )
 *
 * and of its backward pass, for one MI355X (gfx950).
 *
 * The paper (section "SOL principle") replaces step 1 of the training loop, the model
 * forward pass, and step 3, the backward pass, by compiled code in which connected layers
 * are merged (section "SOL architecture", the paragraph on grouping and layer merging);
 * the framework keeps only memory allocation, the loss and the weight update.  For a
 * ResNet-50-style network (the paper's benchmark model, section "SOL Benefits") the merged
 * groups are exactly these blocks.  sol_block_fwd is step 1 for one block, sol_block_bwd is
 * step 3 for one block.  The paper's three generated versions (inference, training forward,
 * training backward) map to: fwd whose y is discarded later, fwd whose y is kept, bwd.
 *
 * Layout (all tensors dense, no strides):
 *   activations  NHWC   x[N][H][W][C_in],  y / residual / dy / dres[N][Ho][Wo][C_out],
 *                       dx / dx_addend[N][H][W][C_in]
 *   weights      KRSC   W / dW[C_out][KH][KW][C_in]
 *   Ho = (H + 2*pad - KH) / stride + 1, likewise Wo.   Cross-correlation, no bias,
 *   dilation 1, groups 1, symmetric zero padding.
 * Types:
 *   SOL_BF16: x, W, residual, y, dy, dx, dres, dx_addend are bfloat16; scale, shift, dW,
 *             dscale, dshift and every accumulator are float32.  One rounding (to nearest
 *             even) at each bf16 store.
 *   SOL_F32 : everything float32.
 * Ownership: every pointer is a DEVICE pointer owned by the caller (16-byte aligned); the
 *   library never allocates, frees or keeps device memory, never synchronises, and enqueues
 *   only on the stream passed in (a hipStream_t, 0 = the null stream).  Inputs are read-only;
 *   outputs are overwritten.  Outputs may not alias inputs (dx_addend == dx is allowed).
 * Errors: every entry point returns 0 on success or a negative sol_status; nothing is
 *   thrown, printed or aborted.  Argument checks are host-only and happen before any HIP
 *   call, so a call that fails validation never touches the device.
 * Thread safety: re-entrant; calls that share an output or workspace buffer race.
 */
#ifndef SOL_BLOCK_H
#define SOL_BLOCK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SOL_API __attribute__((visibility("default")))

typedef enum { SOL_F32 = 0, SOL_BF16 = 1 } sol_dtype;

enum {
    SOL_RELU = 1u << 0,          /* ReLU is the last operation of the block               */
    SOL_DW_ACCUMULATE = 1u << 1  /* bwd adds into dW / dscale / dshift instead of storing */
};

typedef enum {
    SOL_OK = 0,
    SOL_ERR_NULL = -1,        /* a required pointer is NULL                                 */
    SOL_ERR_SHAPE = -2,       /* non-positive size, stride < 1, pad < 0, empty output, ...  */
    SOL_ERR_ALIGN = -3,       /* a pointer is not 16-byte aligned                           */
    SOL_ERR_UNSUPPORTED = -4, /* unknown dtype / flag bits, tensor beyond 2^31-1 elements   */
    SOL_ERR_WORKSPACE = -5,   /* workspace missing or smaller than sol_block_workspace_bytes */
    SOL_ERR_LAUNCH = -6,      /* the HIP runtime reported an error at launch                */
    SOL_ERR_SCRATCH_LIMIT = -7 /* sol_block_bwd_noalloc: the call needs more scratch than the built-in buffer holds */
} sol_status;

typedef struct {
    int32_t N, H, W, C_in;   /* x : [N][H][W][C_in]                 */
    int32_t C_out, KH, KW;   /* W : [C_out][KH][KW][C_in]           */
    int32_t stride, pad;     /* same in h and w                     */
    int32_t dtype;           /* sol_dtype                           */
    uint32_t flags;          /* SOL_RELU | SOL_DW_ACCUMULATE        */
} sol_block_desc;

enum { SOL_PASS_FWD = 0, SOL_PASS_BWD = 1 };

/*
 * Step 1 for one block (training-forward and inference versions are the same call):
 *   z = conv(x, W);  v = scale[c]*z + shift[c] (+ residual);  y = ReLU ? max(v, 0) : v.
 * residual may be NULL.  ws / ws_bytes: at least sol_block_workspace_bytes(desc, SOL_PASS_FWD)
 * bytes (may be NULL when that is 0).
 */
SOL_API int sol_block_fwd(const sol_block_desc* desc, const void* x, const void* W, const float* scale,
                  const float* shift, const void* residual, void* y, void* ws, size_t ws_bytes,
                  void* hip_stream);

/*
 * Step 3 for one block.  With g = ReLU ? (y > 0 ? dy : 0) : dy  (the block's own stored
 * output y decides the mask, which is why training must keep y between the passes -- the
 * paper's remark on intermediate results in its section on memory consumption):
 *   dx[n,hi,wi,ci]  = sum_{kh,kw,co} g[n,ho,wo,co] * scale[co] * W[co,kh,kw,ci]   (+ addend)
 *   dW[co,kh,kw,ci] = scale[co] * sum_{n,ho,wo} g[n,ho,wo,co] * x[n,hi,wi,ci]
 *   dshift[co]      = sum g[.,co]          dscale[co] = sum g[.,co] * conv(x,W)[.,co]
 * Nullable: dx (skips the data gradient altogether), dres, dx_addend, dx_addend_mask, dx_mask;
 * dW, dscale and dshift may be NULL together (skips the weight branch: the split weight-gradient
 * GEMM and its reduction); at least one of dx, dres, dW must be given.  The data branch and the
 * weight branch of ONE block read the same inputs and use disjoint parts of the workspace, so a
 * caller may issue them as two calls on two streams (one with dW = NULL, one with dx = dres =
 * NULL) sharing one workspace.  That holds for two calls with the same descriptor only: where the
 * parts lie depends on the descriptor, so calls for different blocks that may overlap in time
 * (a weight branch still running on a side stream while the next block starts) need a workspace
 * each.
 *   dres            out, [N][Ho][Wo][C_out]: g itself (the gradient of the residual input).
 *   dx_addend       in,  [N][H][W][C_in]: added to dx in the epilogue (shortcut gradients).
 *   dx_addend_mask  in,  same shape as dx_addend: when given, only elements whose mask value
 *                   is > 0 are added (lets a shortcut pass dy of the tail block together with
 *                   that block's y instead of materialising its g).
 *   dx_mask         in,  same shape as dx: when given, dx is stored as 0 wherever the mask value
 *                   is <= 0 (applied after the addend).  Passing the block input -- the stored
 *                   output of the ReLU block that produced it -- hands the upstream block a
 *                   gradient that is already masked, so that block can be called without
 *                   SOL_RELU and without its y: the mask costs one read here instead of one read
 *                   in each of the upstream block's two gradient kernels.
 * scale is required (dx and dW carry it); shift never enters a gradient.
 * Results do not depend on run or launch order (no floating-point atomics).
 */
SOL_API int sol_block_bwd(const sol_block_desc* desc, const void* dy, const void* x, const void* W,
                  const void* y, void* dx, float* dW, float* dscale, float* dshift,
                  const float* scale, void* dres, const void* dx_addend,
                  const void* dx_addend_mask, const void* dx_mask, void* ws, size_t ws_bytes,
                  void* hip_stream);

/*
 * sol_block_bwd for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as sol_block_bwd without ws / ws_bytes: the scratch (re-packed
 * weights, split partial sums) lives in a buffer of SOL_NOALLOC_SCRATCH_BYTES bytes that is part of
 * the library's code object, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing.  SOL_ERR_SCRATCH_LIMIT when sol_block_workspace_bytes(desc, SOL_PASS_BWD) exceeds
 * that size (nothing is launched then); sol_block_bwd_noalloc_limit() returns the size.  The GPU the
 * stream belongs to must be the current device of the calling thread.  Every call on a GPU uses that
 * GPU's one buffer and finds the previous call's contents in it (the kernels overwrite what they read
 * back): calls that may overlap in time on one GPU -- two streams, two threads -- race; order them.
 */
#define SOL_NOALLOC_SCRATCH_BYTES (40u << 20)
SOL_API int sol_block_bwd_noalloc(const sol_block_desc* desc, const void* dy, const void* x, const void* W,
                          const void* y, void* dx, float* dW, float* dscale, float* dshift,
                          const float* scale, void* dres, const void* dx_addend,
                          const void* dx_addend_mask, const void* dx_mask, void* hip_stream);
SOL_API size_t sol_block_bwd_noalloc_limit(void);

/* Bytes of caller-provided scratch the given pass needs for this descriptor (0 if the
 * descriptor is invalid: the pass itself then reports the error).  The answer depends on every
 * field of the descriptor, flags included (a backward pass that masks dy itself keeps the masked
 * gradient in the workspace): ask with the descriptor the call will carry. */
SOL_API size_t sol_block_workspace_bytes(const sol_block_desc* desc, int pass);

/*
 * Launch plans.  The paper tunes every layer on its own when a network is compiled (section "SOL
 * architecture", the auto-tuning of the layer implementations).  Here the library picks tile
 * shape, pipeline depth and the split of the weight gradient from the problem size, with thresholds
 * measured over the benchmark network's layers; a caller may instead time the few candidates once
 * per layer shape and install the winner.  A plan is looked up by the descriptor's shape, stride,
 * padding and dtype (flags do not matter) and by the kernel it steers:
 *   SOL_PLAN_FWD    forward GEMM:        tile, stages
 *   SOL_PLAN_DGRAD  data-gradient GEMM:  tile, stages
 *   SOL_PLAN_WGRAD  weight gradient:     splits (workgroups along N*Ho*Wo), stages
 * tile: 0 = 128 pixels x 128 channels, 1 = 128 x 64, 2 = 64 x 64, 3 = 256 x 128 (stages 2 or 3
 * only), 4 = 128-pixel panel kept in LDS while the workgroup walks over several 128-channel tiles
 * (1x1 / stride 1 layers with 64 .. 256 input channels and a multiple of 128 output channels, no
 * gate on the addend; ignored elsewhere; stages not used), -1 = library's choice.  stages: 2, 3 or
 * 4 slices in flight, 0 = library's choice.
 * splits: 0 = library's choice; the workspace size of the backward pass depends on it, so install
 * plans before asking sol_block_workspace_bytes.  Plans only apply where the pipelined bf16 kernels
 * run; elsewhere they are ignored.  They change speed, never which result is correct: forward and
 * data gradient do not depend on the plan at all, the weight gradient only in the order of its fp32
 * partial sums.  Host-only calls, safe from any thread (a small table behind a mutex).
 */
enum { SOL_PLAN_FWD = 0, SOL_PLAN_DGRAD = 1, SOL_PLAN_WGRAD = 2 };
typedef struct {
    int32_t tile;
    int32_t stages;
    int32_t splits;
} sol_plan;
/* Installs (plan != NULL) or removes (plan == NULL) the plan of one kernel of one layer shape.
 * SOL_ERR_UNSUPPORTED for values outside the ranges above, SOL_ERR_SHAPE etc. for a bad descriptor. */
SOL_API int sol_block_set_plan(const sol_block_desc* desc, int which, const sol_plan* plan);
/* The installed plan, or {-1, 0, 0} when the library decides by itself. */
SOL_API int sol_block_get_plan(const sol_block_desc* desc, int which, sol_plan* out);
/* Removes every installed plan. */
SOL_API void sol_clear_plans(void);

/* Tuning-experiment overrides (environment variables SOL_IGEMM_FAST, SOL_FAST_TILE, SOL_FAST_STAGES,
 * SOL_IGEMM_TILE, SOL_WGRAD_FAST, SOL_WGRAD_SPLITS, SOL_WGRAD_STAGES, ...: they win over installed
 * plans) are read once, by the first call that looks at one, not per call.  This reads them again;
 * for tests and sweeps that change the environment of a running process.  Host-only. */
SOL_API void sol_reload_overrides(void);

/* Static, NUL-terminated description of a status code. */
SOL_API const char* sol_status_string(int status);

/*
 * Glue that the paper leaves to the framework (loss, section "SOL principle") or that is not
 * a convolution (the stem max-pool of the benchmark network); provided so that a whole
 * training step can run without any framework kernel.  Same pointer / stream rules.
 */

/* dy = sign(y - t) / numel (sign(0) = 0): gradient of the mean absolute error.  With mask_by_y != 0
 * the result is additionally 0 wherever y <= 0, i.e. already masked by the ReLU that produced y. */
SOL_API int sol_l1_loss_grad(int32_t dtype, const void* y, const void* t, void* dy, int64_t numel,
                     int32_t mask_by_y, void* hip_stream);

/* Max-pool k x k / stride / pad over NHWC (padding never wins). */
SOL_API int sol_maxpool_fwd(int32_t dtype, const void* x, void* y, int32_t N, int32_t H, int32_t W,
                    int32_t C, int32_t k, int32_t stride, int32_t pad, void* hip_stream);

/*
 * Prepared sequences.  The paper's compiled network is one library call that runs a static schedule
 * (section "SOL architecture": the generated library holds the whole execution pipeline; section on
 * memory consumption: the schedule is static).  A sequence is that schedule for this library: the
 * caller records the block calls of a pass once, with their final buffers, and sol_sequence_run then
 * issues calls [first, first + count) in order on one stream without returning to the caller between
 * launches.  Recording validates nothing and touches no device; every recorded call behaves exactly
 * like the entry point it names when it is run (same checks, same errors: run stops at the first
 * failing call and returns its status).  The sequence keeps copies of the descriptors and of the
 * pointer VALUES only; the buffers stay the caller's and must outlive the runs.  A sequence is a
 * host object (sol_sequence_create / sol_sequence_destroy); running one sequence from two threads at
 * once is safe only if the recorded calls may overlap (see the workspace rule of sol_block_bwd).
 * tag: any number; it labels the launches of that call in a launch trace.
 */
typedef struct sol_sequence sol_sequence;
SOL_API sol_sequence* sol_sequence_create(void);                 /* NULL when out of host memory */
SOL_API void sol_sequence_destroy(sol_sequence* seq);            /* NULL is allowed */
SOL_API int32_t sol_sequence_length(const sol_sequence* seq);
SOL_API int sol_sequence_add_fwd(sol_sequence* seq, const sol_block_desc* desc, const void* x, const void* W,
                         const float* scale, const float* shift, const void* residual, void* y, void* ws,
                         size_t ws_bytes, int32_t tag);
SOL_API int sol_sequence_add_bwd(sol_sequence* seq, const sol_block_desc* desc, const void* dy, const void* x,
                         const void* W, const void* y, void* dx, float* dW, float* dscale, float* dshift,
                         const float* scale, void* dres, const void* dx_addend, const void* dx_addend_mask,
                         const void* dx_mask, void* ws, size_t ws_bytes, int32_t tag);
SOL_API int sol_sequence_add_l1_loss_grad(sol_sequence* seq, int32_t dtype, const void* y, const void* t, void* dy,
                                  int64_t numel, int32_t mask_by_y, int32_t tag);
SOL_API int sol_sequence_add_maxpool(sol_sequence* seq, int32_t dtype, const void* x, void* y, int32_t N, int32_t H,
                             int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, int32_t tag);
SOL_API int sol_sequence_run(const sol_sequence* seq, int32_t first, int32_t count, void* hip_stream);

/*
 * Launch trace: GPU time of every kernel launch the library makes, in launch order, without an external
 * profiler (the per-layer timing that the paper's auto-tuning relies on, section "SOL architecture").
 * Between sol_trace_start and sol_trace_stop every launch carries a start and a stop event of its own,
 * stamped from the dispatch itself (no barrier between kernels, so the step runs as it does untraced and
 * the times are the kernels' execution times, as a profiler reports them).  sol_trace_stop waits for the
 * launches and returns, per launch in launch order: its kind, the tag that was current when it was issued
 * (sol_trace_tag, or the tag of the sequence call), its execution time and its start relative to the
 * first traced launch, both in microseconds.  capacity of sol_trace_start = launches to provide events
 * for; launches beyond it run untraced.  The events are created by sol_trace_start (the only place in the
 * library that creates HIP objects) and kept for later traces.
 * One trace at a time, all calls traced must use one stream; not for use under graph capture.
 * The two ..._REDUCE kinds are data-gradient launches of sol_block_bwd that also carry the reduction of the same
 * call's split weight gradient (as extra workgroups), which then is no launch of its own.
 */
enum {
    SOL_TRACE_OTHER = 0, SOL_TRACE_IGEMM, SOL_TRACE_IGEMM_GENERAL, SOL_TRACE_WGRAD, SOL_TRACE_WGRAD_GENERAL,
    SOL_TRACE_WGRAD_REDUCE, SOL_TRACE_PACK, SOL_TRACE_UNTOUCHED, SOL_TRACE_MASKED_COPY, SOL_TRACE_SMALLC_PREPARE,
    SOL_TRACE_SMALLC_FWD, SOL_TRACE_SMALLC_WGRAD, SOL_TRACE_DIRECT, SOL_TRACE_L1_GRAD, SOL_TRACE_MAXPOOL,
    SOL_TRACE_IGEMM_PANEL, SOL_TRACE_IGEMM_REDUCE, SOL_TRACE_IGEMM_PANEL_REDUCE
};
typedef struct {
    int32_t kind;   /* SOL_TRACE_* */
    int32_t tag;
    float us;       /* execution time of the launch            */
    float start_us; /* its start, counted from the first launch */
} sol_trace_entry;
SOL_API int sol_trace_start(int32_t capacity);
SOL_API void sol_trace_tag(int32_t tag);
SOL_API int sol_trace_stop(sol_trace_entry* out, int32_t capacity, int32_t* count);
SOL_API const char* sol_trace_kind_name(int32_t kind);

#ifdef __cplusplus
}
#endif
#endif /* SOL_BLOCK_H */
