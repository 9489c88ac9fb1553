// C-ABI of the fused block: argument validation (host only, before any HIP call), launch
// planning (tile shape, split count, workspace layout) and the calls into the kernels.
#include <limits.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <map>
#include <mutex>

#include "../../include/sol_block.h"
#include "classes.h"
#include "launch.h"
#include "pack_tile.h"
#include "reduce_rows.h"

namespace sol {
namespace {

constexpr size_t kAlign = 256;
int builtin_scratch_address(void** out);      // device address of this GPU's built-in scratch array
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

struct Geometry {
    int Ho, Wo;
    long long M, K;
    long long x_elems, y_elems, w_elems;
};

int check_desc(const sol_block_desc* d, Geometry* g) {
    if (!d) return SOL_ERR_NULL;
    if (d->dtype != SOL_F32 && d->dtype != SOL_BF16) return SOL_ERR_UNSUPPORTED;
    if (d->flags & ~(uint32_t)(SOL_RELU | SOL_DW_ACCUMULATE)) return SOL_ERR_UNSUPPORTED;
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C_in < 1 || d->C_out < 1 || d->KH < 1 || d->KW < 1 ||
        d->stride < 1 || d->pad < 0)
        return SOL_ERR_SHAPE;
    if (d->H + 2 * (long long)d->pad < d->KH || d->W + 2 * (long long)d->pad < d->KW) return SOL_ERR_SHAPE;
    g->Ho = (d->H + 2 * d->pad - d->KH) / d->stride + 1;
    g->Wo = (d->W + 2 * d->pad - d->KW) / d->stride + 1;
    g->M = (long long)d->N * g->Ho * g->Wo;
    g->K = (long long)d->KH * d->KW * d->C_in;
    g->x_elems = (long long)d->N * d->H * d->W * d->C_in;
    g->y_elems = g->M * d->C_out;
    g->w_elems = g->K * d->C_out;
    const long long lim = 0x7fffffffLL;
    if (g->x_elems > lim || g->y_elems > lim || g->w_elems > lim) return SOL_ERR_UNSUPPORTED;
    return SOL_OK;
}

// hipGetLastError() reports the last error of ANY earlier HIP call on this thread (the caller's
// framework included); drop it so that the check after our launches sees only our own.
inline void clear_stale_error() { (void)hipGetLastError(); }

// Tuning-experiment overrides from the environment.  They are read once (at the first call that needs one,
// or when sol_reload_overrides() asks for it), never per call: every getenv walks the whole environment, and a
// backward call used to make some fifteen of them.
enum Knob {
    K_IGEMM_TILE, K_IGEMM_FAST, K_FAST_TILE, K_FAST_SHORTK, K_FAST_MANY, K_FAST_STAGES, K_WGRAD_SPLITS, K_WGRAD_TARGET,
    K_SMALLC, K_FILL_UNTOUCHED, K_WGRAD_FAST, K_PACK_FUSED, K_WGRAD_STAGES, K_PREMASK, K_PANEL, K_PANEL_TILES,
    K_REDUCE_RIDES, K_COUNT
};
const char* const kKnobNames[K_COUNT] = {
    "SOL_IGEMM_TILE", "SOL_IGEMM_FAST", "SOL_FAST_TILE", "SOL_FAST_SHORTK", "SOL_FAST_MANY", "SOL_FAST_STAGES",
    "SOL_WGRAD_SPLITS", "SOL_WGRAD_TARGET", "SOL_SMALLC", "SOL_FILL_UNTOUCHED", "SOL_WGRAD_FAST", "SOL_PACK_FUSED",
    "SOL_WGRAD_STAGES", "SOL_PREMASK", "SOL_PANEL", "SOL_PANEL_TILES", "SOL_REDUCE_RIDES"};
constexpr int kKnobUnset = INT32_MIN;
std::atomic<int> g_knobs[K_COUNT];
std::atomic<bool> g_knobs_loaded{false};
std::mutex g_knob_mutex;
void load_knobs() {
    std::lock_guard<std::mutex> lock(g_knob_mutex);
    for (int k = 0; k < K_COUNT; ++k) {
        const char* v = getenv(kKnobNames[k]);
        g_knobs[k].store(v && *v ? atoi(v) : kKnobUnset, std::memory_order_relaxed);
    }
    g_knobs_loaded.store(true, std::memory_order_release);
}
int knob(Knob k, int fallback) {
    if (!g_knobs_loaded.load(std::memory_order_acquire)) load_knobs();
    const int v = g_knobs[k].load(std::memory_order_relaxed);
    return v == kKnobUnset ? fallback : v;
}

// ---- installed launch plans (sol_block_set_plan): shape -> tile / ring depth / split count ----
struct PlanKey {
    int32_t v[11];
    bool operator<(const PlanKey& o) const { return memcmp(v, o.v, sizeof v) < 0; }
};
PlanKey plan_key(const sol_block_desc* d, int which) {
    return PlanKey{{d->N, d->H, d->W, d->C_in, d->C_out, d->KH, d->KW, d->stride, d->pad, d->dtype, which}};
}
std::mutex g_plan_mutex;
std::map<PlanKey, sol_plan> g_plans;
std::atomic<int> g_plan_count{0};              // lets the common case (no plans) skip the lock
sol_plan installed_plan(const sol_block_desc* d, int which) {
    sol_plan out{-1, 0, 0};
    if (g_plan_count.load(std::memory_order_acquire) == 0) return out;
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    auto it = g_plans.find(plan_key(d, which));
    if (it != g_plans.end()) out = it->second;
    return out;
}

// Largest tile that still yields about one workgroup per compute unit; small problems fall
// back to the smallest tile.  SOL_IGEMM_TILE overrides (tuning experiments).
int pick_igemm_tile(const long long* class_rows, int ncls, int Nc) {
    const int forced = knob(K_IGEMM_TILE, -1);
    if (forced >= 0 && forced <= 3) return forced;
    const int order_wide[4] = {1, 0, 2, 3};
    const int order_narrow[2] = {2, 3};
    const int* order = Nc > 64 ? order_wide : order_narrow;
    const int n = Nc > 64 ? 4 : 2;
    for (int i = 0; i < n; ++i) {
        int bp, bc;
        igemm_tile_shape(order[i], &bp, &bc);
        long long tiles = 0;
        for (int c = 0; c < ncls; ++c) tiles += (class_rows[c] + bp - 1) / bp;
        tiles *= (Nc + bc - 1) / bc;
        if (tiles >= 192) return order[i];
    }
    return order[n - 1];
}

// A pipelined or panel launch of `gemm_wgs` workgroups (one per compute unit at a time) can carry the split
// reduction of the same block's weight gradient along, as workgroups behind its own: as many as its last wave
// leaves compute units idle, so that the reduction runs beside the tiles instead of after them.  Returns 0 when
// fewer than 32 are idle (the reduction then stays a launch of its own).  The two smaller tiles run several workgroups
// per compute unit in many waves: there the riders fill the launch's tail, one per compute unit at most and no more
// than there are passes over the rows.  SOL_REDUCE_RIDES: 0 never, n > 1 that many.
int reduce_rider_blocks(int gemm_wgs, bool small_tile, const ReduceParams* rider) {
    const int forced = knob(K_REDUCE_RIDES, 1);
    if (!rider || forced == 0 || gemm_wgs <= 0 || !reduce_can_ride(*rider)) return 0;
    if (forced > 1) return forced < 1024 ? forced : 1024;
    if (small_tile) {
        const int rows_per_pass = rider->K <= 256 ? 4 : (rider->K <= 512 ? 2 : 1);
        const int passes = (rider->C_out + rows_per_pass - 1) / rows_per_pass;
        return passes < 256 ? passes : 256;
    }
    const int idle = (256 - gemm_wgs % 256) % 256;
    return idle >= 32 ? idle : 0;
}

// Fills tile-dependent fields of the launch (tile counts, class offsets) and launches either the
// pipelined kernel (source channels % 64 == 0, output channels % 8 == 0, no mask on the gathered
// operand) or the general one.  SOL_IGEMM_FAST=0 forces the general kernel; SOL_FAST_TILE /
// SOL_FAST_STAGES override the pipelined kernel's tile and ring depth (tuning experiments).
// `rider`: a split reduction the launch may carry along (see above); *rode tells whether it did.
int run_igemm(IgemmParams& p, const long long* rows, bool mask, const sol_plan& tuned, hipStream_t stream,
              const ReduceParams* rider = nullptr, bool* rode = nullptr) {
    if (rode) *rode = false;
    auto attach = [&](bool small_tile) {            // p.total_tiles is final
        p.red_blocks = reduce_rider_blocks(p.total_tiles, small_tile, rider);
        if (p.red_blocks > 0) p.red = *rider;
        if (rode) *rode = p.red_blocks > 0;
        return p.red_blocks > 0;
    };
    bool few_taps = true;                       // the pipelined kernel keeps one validity bit per tap
    for (int c = 0; c < p.ncls; ++c) few_taps = few_taps && p.cls[c].Th * p.cls[c].Tw <= 32;
    // the pipelined kernel starts its buffer descriptor a few image rows before the gathered tensor (the reach of the
    // taps around a pixel); tensor plus that reach must stay below 2^32 bytes
    long long reach = 0;
    for (int c = 0; c < p.ncls; ++c) {
        const RowClass& rc = p.cls[c];
        const long long first = ((long long)rc.h_off * p.Ws + rc.w_off) * p.Cs * 2;
        const long long last = (((long long)(rc.Th - 1) * p.Ws + (rc.Tw - 1)) * rc.tap_step) * p.Cs * 2;
        const long long m = (first < 0 ? -first : 0) + (last < 0 ? -last : 0);
        if (m > reach) reach = m;
    }
    const bool addressable = (long long)p.src_bytes + reach <= 0xffffffffLL && reach <= 0x7fffffffLL;
    const bool fast_ok = !mask && few_taps && addressable && (p.Cs % 64) == 0 && (p.Nc % 8) == 0 &&
                         knob(K_IGEMM_FAST, 1) != 0;
    int bp, bc, tile = 0, stages = 0;
    bool many_tiles = false;
    // 1x1 / stride 1 with a short reduction and a wide output: a workgroup keeps its pixel panel in LDS and walks over
    // several channel tiles (tile code 4)
    const bool panel_ok = fast_ok && knob(K_PANEL, 1) != 0 && igemm_panel_eligible(p);
    if (fast_ok) {
        long long slices = 0;
        for (int c = 0; c < p.ncls; ++c) {
            const long long s = (long long)p.cls[c].Th * p.cls[c].Tw * (p.Cs / 64);
            if (s > slices) slices = s;
        }
        tile = knob(K_FAST_TILE, -1);
        if (tile < 0 || tile > 4) tile = tuned.tile;              // an installed plan; the environment wins (experiments)
        if (tile == 4 && !panel_ok) tile = -1;                    // a plan for the panel kernel on a launch it cannot run
        if (tile < 0 || tile > 4) {
            // 128 x 128 unless that leaves most compute units idle or the GEMM is narrow
            long long t128 = 0;
            for (int c = 0; c < p.ncls; ++c) t128 += (rows[c] + 127) / 128;
            t128 *= (p.Nc + 127) / 128;
            tile = p.Nc <= 64 ? 1 : (t128 >= 160 ? 0 : 1);
            // short reductions are dominated by per-workgroup latency (prologue, epilogue): many small
            // workgroups per compute unit hide it better than few large ones
            if (slices <= knob(K_FAST_SHORTK, 4) && t128 >= 512) tile = 2;
            // many tiles per compute unit: 128 x 64 tiles with two stages leave room for three workgroups per
            // compute unit, whose prologues and epilogues overlap (measured over the ResNet-50 layer shapes:
            // best or within a few percent of best from ~3 tiles of 128 x 128 per compute unit upwards)
            many_tiles = t128 >= knob(K_FAST_MANY, 700) * (slices <= 4 ? 2 : 1);   // short reductions: 64 x 64 holds up longer
            if (many_tiles) tile = 1;
            long long t = 0;
            igemm_fast_tile_shape(tile, &bp, &bc);
            for (int c = 0; c < p.ncls; ++c) t += (rows[c] + bp - 1) / bp;
            t *= (p.Nc + bc - 1) / bc;
            if (t < 160) tile = 2;
            // the panel kernel where its launch is one wave of workgroups that fills most of the chip
            if (panel_ok) {
                const long long panels = (rows[0] + 127) / 128;
                long long groups = 256 / (panels > 0 ? panels : 1);
                if (groups > p.Nc / 128) groups = p.Nc / 128;
                if (panels <= 256 && panels * groups >= 160) tile = 4;
            }
        }
        if (tile == 4) {
            plan_igemm_panel(p, knob(K_PANEL_TILES, 0));
            trace_point(stream, attach(false) ? SOL_TRACE_IGEMM_PANEL_REDUCE : SOL_TRACE_IGEMM_PANEL);
            return launch_igemm_panel(p, stream) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
        }
        stages = knob(K_FAST_STAGES, 0);
        if (stages < 2 || stages > 4) stages = tuned.stages;
        if (stages < 2 || stages > 4) stages = (slices <= 4 || many_tiles) ? 2 : (slices <= 8 ? 3 : 4);
        if (tile == 3 && stages > 3) stages = 3;
        igemm_fast_tile_shape(tile, &bp, &bc);
    } else {
        tile = pick_igemm_tile(rows, p.ncls, p.Nc);
        igemm_tile_shape(tile, &bp, &bc);
    }
    p.tiles_c = (p.Nc + bc - 1) / bc;
    int tiles_p = 0;
    for (int c = 0; c < p.ncls; ++c) {
        RowClass& rc = p.cls[c];
        const bool lin_src = rc.Th == 1 && rc.Tw == 1 && rc.h_mul == 1 && rc.w_mul == 1 && rc.h_off == 0 &&
                             rc.w_off == 0 && rc.Rh == p.Hs && rc.Rw == p.Ws;
        const bool lin_out = rc.oh_mul == 1 && rc.ow_mul == 1 && rc.oh_off == 0 && rc.ow_off == 0 &&
                             rc.Rh == p.Hout && rc.Rw == p.Wout;
        rc.linear = (lin_src ? 1 : 0) | (lin_out ? 2 : 0);
        rc.div_img = make_fast_div((uint32_t)(rc.Rh * rc.Rw));
        rc.div_rw = make_fast_div((uint32_t)rc.Rw);
        p.cls[c].tile_begin = tiles_p;
        tiles_p += (int)((rows[c] + bp - 1) / bp);
    }
    p.total_tiles = tiles_p * p.tiles_c;
    hipError_t e;
    const bool rides = fast_ok && attach(tile == 1 || tile == 2);
    trace_point(stream, rides ? SOL_TRACE_IGEMM_REDUCE : fast_ok ? SOL_TRACE_IGEMM : SOL_TRACE_IGEMM_GENERAL);
    if (fast_ok) e = launch_igemm_fast(p, tile, stages, stream);
    else e = launch_igemm(p, tile, (p.Cs % 8) == 0, mask, stream);
    return e == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
}

struct BwdPlan {
    int splits, m_per_split, tiles_k, tiles_c;
    size_t wpack_off, part_off, dshift_off, total;
    // few-input-channel layers: channel-padded image and per-workgroup partials of their own weight-gradient kernel
    bool smallc;
    int sc_parts;
    size_t sc_xp_off, sc_part_off;
    // a block that masks dy itself (SOL_RELU): the masked gradient, written once by an element-wise launch so that
    // both gradient GEMMs take the pipelined kernels (which gather their operands without looking at y)
    bool premask;
    size_t gmask_off;
};

// channel counts the 16-byte operand pieces of the bf16 kernels need
inline bool bf16_vector_shape(const sol_block_desc* d) {
    return d->dtype == SOL_BF16 && (d->C_in % 8) == 0 && (d->C_out % 8) == 0;
}

BwdPlan plan_bwd(const sol_block_desc* d, const Geometry& g) {
    BwdPlan b{};
    if (d->dtype == SOL_F32) {
        b.splits = 1;
        b.m_per_split = (int)g.M;
        b.wpack_off = 0;
        b.part_off = 0;
    } else {
        b.tiles_k = (int)((g.K + 127) / 128);
        b.tiles_c = (d->C_out + 127) / 128;
        const long long tiles = (long long)b.tiles_k * b.tiles_c;
        const long long max_splits = (g.M + 127) / 128;
        long long want = knob(K_WGRAD_SPLITS, 0);
        if (want <= 0) want = installed_plan(d, SOL_PLAN_WGRAD).splits;
        if (want <= 0) {
            // Workgroups aimed at (per-layer timing over the benchmark network's layers): the 1x1 / stride 1
            // kernel runs three stages deep, one workgroup per compute unit, and is fastest with one wave of
            // 256 workgroups; the gathering kernel runs two stages deep, two workgroups per compute unit: 512.
            const bool linear = d->KH == 1 && d->KW == 1 && d->stride == 1 && d->pad == 0;
            const long long target = knob(K_WGRAD_TARGET, linear ? 256 : 512);
            want = (target + tiles - 1) / tiles;
            // keep the fp32 partials below ~64 MiB
            const long long cap = (64LL << 20) / (g.w_elems * 4 > 0 ? g.w_elems * 4 : 1);
            if (want > cap) want = cap;
        }
        if (want < 1) want = 1;
        if (want > max_splits) want = max_splits;
        long long mps = (g.M + want - 1) / want;
        mps = (mps + 127) / 128 * 128;
        b.m_per_split = (int)mps;
        b.splits = (int)((g.M + mps - 1) / mps);
        b.wpack_off = 0;
        b.part_off = align_up((size_t)g.w_elems * 2);
    }
    b.dshift_off = b.part_off + align_up((size_t)b.splits * g.w_elems * 4);
    b.total = b.dshift_off + align_up((size_t)b.splits * d->C_out * 4);
    b.smallc = d->dtype == SOL_BF16 && smallc_wgrad_supported(d->C_in, d->C_out, d->KH, d->KW, d->stride) &&
               knob(K_SMALLC, 1) != 0;
    if (b.smallc) {
        b.sc_parts = smallc_wgrad_parts(d->N, g.Ho, g.Wo);
        b.sc_xp_off = b.total;
        b.sc_part_off = b.sc_xp_off + align_up(smallc_padded_image_bytes(d->N, d->H, d->W));
        b.total = b.sc_part_off + align_up(smallc_wgrad_partial_bytes(b.sc_parts));
    }
    b.premask = (d->flags & SOL_RELU) != 0 && d->dtype == SOL_BF16 && (bf16_vector_shape(d) || b.smallc) &&
                knob(K_PREMASK, 1) != 0;
    if (b.premask) {
        b.gmask_off = b.total;
        b.total += align_up((size_t)g.y_elems * 2);
    }
    return b;
}

// Forward workspace: only the few-input-channel kernel needs one (channel-padded image + packed weights).
struct FwdPlan {
    bool smallc;
    size_t xp_off, wp_off, total;
};
FwdPlan plan_fwd(const sol_block_desc* d) {
    FwdPlan f{};
    f.smallc = d->dtype == SOL_BF16 && smallc_fwd_supported(d->C_in, d->C_out, d->KH, d->KW, d->stride) &&
               knob(K_SMALLC, 1) != 0;
    if (f.smallc) {
        f.xp_off = 0;
        f.wp_off = align_up(smallc_padded_image_bytes(d->N, d->H, d->W));
        f.total = f.wp_off + align_up(smallc_packed_weight_bytes(d->KH));
    }
    return f;
}

int fwd_bf16(const sol_block_desc* d, const Geometry& g, const void* x, const void* W, const float* scale,
             const float* shift, const void* residual, void* y, void* ws, hipStream_t stream) {
    const FwdPlan plan = plan_fwd(d);
    if (plan.smallc && !residual) {
        unsigned char* wsb = (unsigned char*)ws;
        SmallCParams sp{(const bf16_t*)x, (bf16_t*)(wsb + plan.xp_off), (const bf16_t*)W, (bf16_t*)(wsb + plan.wp_off),
                        scale, shift, (bf16_t*)y, d->N, d->H, d->W, d->C_in, d->KH, d->KW, d->pad, g.Ho, g.Wo,
                        (d->flags & SOL_RELU) ? 1 : 0};
        trace_point(stream, SOL_TRACE_SMALLC_PREPARE);
        if (launch_smallc_prepare(sp, stream) != hipSuccess) return SOL_ERR_LAUNCH;
        trace_point(stream, SOL_TRACE_SMALLC_FWD);
        return launch_smallc_fwd(sp, stream) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
    }
    IgemmParams p{};
    p.src = (const bf16_t*)x;
    p.src_mask = nullptr;
    p.wmat = (const bf16_t*)W;
    p.out = (bf16_t*)y;
    p.scale = scale;
    p.shift = shift;
    p.addend = (const bf16_t*)residual;
    p.addend_mask = nullptr;
    p.src_bytes = (unsigned)(g.x_elems * 2);
    p.Hs = d->H;
    p.Ws = d->W;
    p.Cs = d->C_in;
    p.Nc = d->C_out;
    p.Hout = g.Ho;
    p.Wout = g.Wo;
    p.relu = (d->flags & SOL_RELU) ? 1 : 0;
    p.ncls = 1;
    RowClass& c = p.cls[0];
    c.rows = (int)g.M;
    c.Rh = g.Ho;
    c.Rw = g.Wo;
    c.h_mul = d->stride;
    c.h_off = -d->pad;
    c.w_mul = d->stride;
    c.w_off = -d->pad;
    c.Th = d->KH;
    c.Tw = d->KW;
    c.tap_step = 1;
    c.oh_mul = 1;
    c.oh_off = 0;
    c.ow_mul = 1;
    c.ow_off = 0;
    c.tile_begin = 0;
    c.b_off = 0;
    const long long rows[1] = {g.M};
    return run_igemm(p, rows, false, installed_plan(d, SOL_PLAN_FWD), stream);
}

int dgrad_bf16(const sol_block_desc* d, const Geometry& g, const void* dy, const void* ymask, const bf16_t* wpack,
               void* dx, const void* addend, const void* addend_mask, const void* dx_mask, hipStream_t stream,
               const ReduceParams* rider = nullptr, bool* rode = nullptr) {
    const int s = d->stride;
    IgemmParams p{};
    const bool relu = ymask != nullptr;          // mask dy by y > 0 while gathering it
    p.src = (const bf16_t*)dy;
    p.src_mask = (const bf16_t*)ymask;
    p.wmat = wpack;
    p.out = (bf16_t*)dx;
    p.scale = nullptr;
    p.shift = nullptr;
    p.addend = (const bf16_t*)addend;
    p.addend_mask = (const bf16_t*)addend_mask;
    p.out_mask = (const bf16_t*)dx_mask;
    p.src_bytes = (unsigned)(g.y_elems * 2);
    p.Hs = g.Ho;
    p.Ws = g.Wo;
    p.Cs = d->C_out;
    p.Nc = d->C_in;
    p.Hout = d->H;
    p.Wout = d->W;
    p.relu = 0;
    long long rows[kMaxClasses];
    int nc = 0;
    // pixels without a tap (1x1 / stride 2: three quarters of dx) are filled at memory speed by a launch of their
    // own; as GEMM tiles without a reduction they cost several times that
    const bool fill_untouched = (d->C_in % 8) == 0 && knob(K_FILL_UNTOUCHED, 1) != 0;
    bool any_untouched = false;
    for (int ph = 0; ph < s; ++ph)
        for (int pw = 0; pw < s; ++pw) {
            const int Rh = d->H > ph ? (d->H - ph + s - 1) / s : 0;
            const int Rw = d->W > pw ? (d->W - pw + s - 1) / s : 0;
            if (Rh == 0 || Rw == 0) continue;
            int fh, fw;
            RowClass& c = p.cls[nc];
            c.Th = class_taps(d->KH, s, d->pad, ph, &fh);
            c.Tw = class_taps(d->KW, s, d->pad, pw, &fw);
            if (c.Th == 0 || c.Tw == 0) {   // no tap reaches these pixels: K = 0, output = addend
                if (fill_untouched) {       // ... written by an element-wise launch instead of GEMM tiles
                    any_untouched = true;
                    continue;
                }
                c.Th = 0;
                c.Tw = 1;
            }
            c.rows = d->N * Rh * Rw;
            c.Rh = Rh;
            c.Rw = Rw;
            c.h_mul = 1;
            c.h_off = (ph + d->pad - fh) / s;
            c.w_mul = 1;
            c.w_off = (pw + d->pad - fw) / s;
            c.tap_step = -1;
            c.oh_mul = s;
            c.oh_off = ph;
            c.ow_mul = s;
            c.ow_off = pw;
            c.b_off = class_weight_offset(d->C_in, d->C_out, d->KH, d->KW, s, d->pad, ph, pw);
            rows[nc] = c.rows;
            ++nc;
        }
    p.ncls = nc;
    if (any_untouched) trace_point(stream, SOL_TRACE_UNTOUCHED);
    if (any_untouched &&
        launch_untouched_pixels(dx, addend, addend_mask, dx_mask, d->N, d->H, d->W, d->C_in, d->KH, d->KW, s, d->pad,
                                stream) != hipSuccess)
        return SOL_ERR_LAUNCH;
    return run_igemm(p, rows, relu, installed_plan(d, SOL_PLAN_DGRAD), stream, rider, rode);
}

}  // namespace
}  // namespace sol

// ---- built-in scratch of the no-allocation backward entry point ---------------------------------------------
// One array per GPU, part of the loaded code object (it exists on every device the library runs on until the
// process ends).  In host code the array's NAME is only a stand-in: the device address is asked for once per
// device, with that device current, and only that address is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[SOL_NOALLOC_SCRATCH_BYTES];

namespace sol {
namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int builtin_scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SOL_ERR_LAUNCH;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return SOL_ERR_LAUNCH;
            }
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return SOL_OK;
}
}  // namespace
}  // namespace sol

using namespace sol;

extern "C" {

SOL_API const char* sol_status_string(int status) {
    switch (status) {
        case SOL_OK: return "ok";
        case SOL_ERR_NULL: return "a required pointer is NULL";
        case SOL_ERR_SHAPE: return "invalid shape, stride or padding";
        case SOL_ERR_ALIGN: return "pointer not 16-byte aligned";
        case SOL_ERR_UNSUPPORTED: return "unsupported dtype, flag or size";
        case SOL_ERR_WORKSPACE: return "workspace missing or too small";
        case SOL_ERR_LAUNCH: return "HIP launch error";
        case SOL_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the no-allocation entry point's built-in buffer holds";
        default: return "unknown status";
    }
}

SOL_API size_t sol_block_workspace_bytes(const sol_block_desc* desc, int pass) {
    Geometry g;
    if (check_desc(desc, &g) != SOL_OK) return 0;
    if (pass == SOL_PASS_FWD) return plan_fwd(desc).total;
    if (pass != SOL_PASS_BWD) return 0;
    return plan_bwd(desc, g).total;
}

SOL_API int sol_block_fwd(const sol_block_desc* desc, const void* x, const void* W, const float* scale, const float* shift,
                  const void* residual, void* y, void* ws, size_t ws_bytes, void* hip_stream) {
    Geometry g;
    if (int e = check_desc(desc, &g); e != SOL_OK) return e;
    if (!x || !W || !scale || !shift || !y) return SOL_ERR_NULL;
    if (misaligned(x) || misaligned(W) || misaligned(scale) || misaligned(shift) || misaligned(y) ||
        misaligned(residual) || misaligned(ws))
        return SOL_ERR_ALIGN;
    const size_t need = plan_fwd(desc).total;
    if (need > 0 && (!ws || ws_bytes < need)) return SOL_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    clear_stale_error();
    if (desc->dtype == SOL_BF16) {
        const int st = fwd_bf16(desc, g, x, W, scale, shift, residual, y, ws, stream);
            return st;
    }
    DirectParams p{};
    p.x = (const float*)x;
    p.W = (const float*)W;
    p.scale = scale;
    p.shift = shift;
    p.res = (const float*)residual;
    p.y = (float*)y;
    p.N = desc->N; p.H = desc->H; p.W_ = desc->W; p.C_in = desc->C_in; p.C_out = desc->C_out;
    p.KH = desc->KH; p.KW = desc->KW; p.stride = desc->stride; p.pad = desc->pad;
    p.Ho = g.Ho; p.Wo = g.Wo; p.relu = (desc->flags & SOL_RELU) ? 1 : 0;
    trace_point(stream, SOL_TRACE_DIRECT);
    const int st = launch_direct_fwd_f32(p, stream) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
    return st;
}

// Both backward entry points: everything after the workspace has been chosen.  scratch_limit > 0 marks the
// built-in buffer of the no-allocation entry point, whose size is a property of the library, not of the call.
static int bwd_common(const sol_block_desc* desc, const void* dy, const void* x, const void* W, const void* y, void* dx,
                      float* dW, float* dscale, float* dshift, const float* scale, void* dres, const void* dx_addend,
                      const void* dx_addend_mask, const void* dx_mask, void* ws, size_t ws_bytes, bool builtin_scratch,
                      void* hip_stream) {
    Geometry g;
    if (int e = check_desc(desc, &g); e != SOL_OK) return e;
    bool relu = (desc->flags & SOL_RELU) != 0;
    if (!dy || !x || !W || !scale) return SOL_ERR_NULL;
    if (dW ? (!dscale || !dshift) : (dscale || dshift)) return SOL_ERR_NULL;   // the three come together
    if (!dW && !dx && !dres) return SOL_ERR_NULL;                              // nothing to compute
    if (relu && !y) return SOL_ERR_NULL;
    if (dx_addend_mask && !dx_addend) return SOL_ERR_NULL;
    if (misaligned(dy) || misaligned(x) || misaligned(W) || misaligned(y) || misaligned(dx) || misaligned(dW) ||
        misaligned(dscale) || misaligned(dshift) || misaligned(scale) || misaligned(dres) ||
        misaligned(dx_addend) || misaligned(dx_addend_mask) || misaligned(dx_mask) || misaligned(ws))
        return SOL_ERR_ALIGN;
    if (desc->dtype == SOL_BF16 && dx && desc->stride * desc->stride > kMaxClasses) return SOL_ERR_UNSUPPORTED;
    const BwdPlan plan = plan_bwd(desc, g);
    if (builtin_scratch) {
        if (plan.total > ws_bytes) return SOL_ERR_SCRATCH_LIMIT;
        if (int e = builtin_scratch_address(&ws); e != SOL_OK) return e;
    }
    if (!ws || ws_bytes < plan.total) return SOL_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    clear_stale_error();
    unsigned char* wsb = (unsigned char*)ws;
    float* partial = (float*)(wsb + plan.part_off);
    float* dshift_partial = (float*)(wsb + plan.dshift_off);
    // A block that masks dy itself: write g = (y > 0 ? dy : 0) once (into dres when the caller wants it anyway) and
    // run everything below on g as a block without ReLU.
    bool dres_done = false;
    if (plan.premask) {
        void* gbuf = dres ? dres : (void*)(wsb + plan.gmask_off);
        trace_point(stream, SOL_TRACE_MASKED_COPY);
        if (launch_masked_copy(desc->dtype, dy, y, gbuf, g.y_elems, stream) != hipSuccess) return SOL_ERR_LAUNCH;
        dy = gbuf;
        relu = false;
        dres_done = dres != nullptr;
    }
    const void* ymask = relu ? y : nullptr;

    auto direct_params = [&]() {
        DirectParams p{};
        p.x = (const float*)x;
        p.W = (const float*)W;
        p.scale = scale;
        p.dy = (const float*)dy;
        p.ymask = (const float*)ymask;
        p.dx = (float*)dx;
        p.addend = (const float*)dx_addend;
        p.addend_mask = (const float*)dx_addend_mask;
        p.dx_mask = (const float*)dx_mask;
        p.G = partial;
        p.dshift_partial = dshift_partial;
        p.N = desc->N; p.H = desc->H; p.W_ = desc->W; p.C_in = desc->C_in; p.C_out = desc->C_out;
        p.KH = desc->KH; p.KW = desc->KW; p.stride = desc->stride; p.pad = desc->pad;
        p.Ho = g.Ho; p.Wo = g.Wo; p.relu = relu ? 1 : 0;
        return p;
    };

    // The re-pack of the weights for the data gradient rides along with the weight-gradient launch (as extra
    // workgroups) when one call computes both branches with the pipelined kernels; else it is a launch of its own.
    const bool bf16_vec = bf16_vector_shape(desc);
    const bool wgrad_pipelined = bf16_vec && !relu && knob(K_WGRAD_FAST, 1) != 0;
    PackParams pk{(const bf16_t*)W, scale, (bf16_t*)(wsb + plan.wpack_off), desc->C_in, desc->C_out, desc->KH,
                  desc->KW, desc->stride, desc->pad};
    const bool pack_rides = dx && dW && wgrad_pipelined && pack_tiled_ok(pk) && knob(K_PACK_FUSED, 1) != 0;

    // The reduction of the split weight gradient in turn may ride along with the data-gradient launch (run_igemm
    // decides); it needs the partial sums of the weight-gradient launch, which therefore goes first.
    ReduceParams rp{};
    rp.partial = partial;
    rp.dshift_partial = dshift_partial;
    rp.W = W;
    rp.scale = scale;
    rp.dW = dW;
    rp.dscale = dscale;
    rp.dshift = dshift;
    rp.C_out = desc->C_out;
    rp.K = (int)g.K;
    rp.splits = plan.splits;
    rp.accumulate = (desc->flags & SOL_DW_ACCUMULATE) ? 1 : 0;
    rp.w_is_bf16 = desc->dtype == SOL_BF16 ? 1 : 0;
    const bool reduce_may_ride = pack_rides;
    bool reduce_rode = false;

    // ---- data branch: shortcut gradient, weight re-pack, data-gradient GEMM ----
    auto data_branch = [&](hipStream_t st) -> int {
        if (dres && !dres_done) {
            trace_point(st, SOL_TRACE_MASKED_COPY);
            if (launch_masked_copy(desc->dtype, dy, ymask, dres, g.y_elems, st) != hipSuccess) return SOL_ERR_LAUNCH;
        }
        if (!dx) return SOL_OK;
        if (desc->dtype == SOL_BF16) {
            if (!pack_rides) trace_point(st, SOL_TRACE_PACK);
            if (!pack_rides && launch_pack_dgrad_weights(pk, st) != hipSuccess) return SOL_ERR_LAUNCH;
            return dgrad_bf16(desc, g, dy, ymask, pk.out, dx, dx_addend, dx_addend_mask, dx_mask, st,
                              reduce_may_ride ? &rp : nullptr, &reduce_rode);
        }
        DirectParams p = direct_params();
        trace_point(st, SOL_TRACE_DIRECT);
        return launch_direct_dgrad_f32(p, st) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
    };

    // ---- weight branch: split weight-gradient GEMM, then the reduction that also finishes dscale, dshift ----
    auto weight_branch = [&](hipStream_t st) -> int {
        if (plan.smallc && !relu) {      // few input channels, gradient already masked: kernels of their own
            bf16_t* xp = (bf16_t*)(wsb + plan.sc_xp_off);
            SmallCParams pp{(const bf16_t*)x, xp, (const bf16_t*)W, nullptr, scale, nullptr, nullptr, desc->N, desc->H,
                            desc->W, desc->C_in, desc->KH, desc->KW, desc->pad, g.Ho, g.Wo, 0};
            trace_point(st, SOL_TRACE_SMALLC_PREPARE);
            if (launch_smallc_prepare(pp, st) != hipSuccess) return SOL_ERR_LAUNCH;
            trace_point(st, SOL_TRACE_SMALLC_WGRAD);
            SmallCWgradParams wp{(const bf16_t*)dy, xp, (const bf16_t*)W, scale, (float*)(wsb + plan.sc_part_off), dW,
                                 dscale, dshift, desc->N, desc->H, desc->W, desc->C_in, desc->KH, desc->KW, desc->pad,
                                 g.Ho, g.Wo, plan.sc_parts, (desc->flags & SOL_DW_ACCUMULATE) ? 1 : 0};
            return launch_smallc_wgrad(wp, st) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
        }
        if (desc->dtype == SOL_BF16) {
            WgradParams wp{};
            wp.dy = (const bf16_t*)dy;
            wp.y = (const bf16_t*)ymask;
            wp.x = (const bf16_t*)x;
            wp.partial = partial;
            wp.dshift_partial = dshift_partial;
            wp.N = desc->N; wp.H = desc->H; wp.W = desc->W; wp.C_in = desc->C_in; wp.C_out = desc->C_out;
            wp.KH = desc->KH; wp.KW = desc->KW; wp.stride = desc->stride; wp.pad = desc->pad;
            wp.Ho = g.Ho; wp.Wo = g.Wo; wp.M = (int)g.M; wp.K = (int)g.K;
            wp.splits = plan.splits; wp.m_per_split = plan.m_per_split;
            wp.tiles_k = plan.tiles_k; wp.tiles_c = plan.tiles_c;
            wp.div_howo = make_fast_div((uint32_t)(g.Ho * g.Wo));
            wp.div_wo = make_fast_div((uint32_t)g.Wo);
            wp.pack = pk;
            wp.pack_blocks = pack_rides ? pack_tile_count(pk) : 0;
            const bool vec = bf16_vec;
            // pipelined kernel when dy needs no mask; SOL_WGRAD_FAST=0 forces the general kernel
            if (wgrad_pipelined) {
                int stages = knob(K_WGRAD_STAGES, 0);
                if (stages < 2 || stages > 4) stages = installed_plan(desc, SOL_PLAN_WGRAD).stages;
                if (stages < 2 || stages > 4)
                    stages = (desc->KH == 1 && desc->KW == 1 && desc->stride == 1 && desc->pad == 0) ? 3 : 2;
                trace_point(st, SOL_TRACE_WGRAD);
                if (launch_wgrad_fast(wp, stages, st) != hipSuccess) return SOL_ERR_LAUNCH;
            } else {
                trace_point(st, SOL_TRACE_WGRAD_GENERAL);
                if (launch_wgrad(wp, vec, relu, st) != hipSuccess) return SOL_ERR_LAUNCH;
            }
        } else {
            DirectParams p = direct_params();
            trace_point(st, SOL_TRACE_DIRECT);
            if (launch_direct_wgrad_f32(p, st) != hipSuccess) return SOL_ERR_LAUNCH;
        }
        if (reduce_may_ride) return SOL_OK;
        trace_point(st, SOL_TRACE_WGRAD_REDUCE);
        return launch_wgrad_reduce(rp, st) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
    };

    // the two branches share only inputs (dy, x, W, scale) and use disjoint parts of the workspace
    int status;
    if (pack_rides) {
        status = weight_branch(stream);
        if (status == SOL_OK) status = data_branch(stream);
        if (status == SOL_OK && !reduce_rode) {
            trace_point(stream, SOL_TRACE_WGRAD_REDUCE);
            if (launch_wgrad_reduce(rp, stream) != hipSuccess) status = SOL_ERR_LAUNCH;
        }
    } else {
        status = data_branch(stream);
        if (status == SOL_OK && dW) status = weight_branch(stream);
    }
    return status;
}

SOL_API int sol_block_bwd(const sol_block_desc* desc, const void* dy, const void* x, const void* W, const void* y, void* dx,
                  float* dW, float* dscale, float* dshift, const float* scale, void* dres, const void* dx_addend,
                  const void* dx_addend_mask, const void* dx_mask, void* ws, size_t ws_bytes, void* hip_stream) {
    return bwd_common(desc, dy, x, W, y, dx, dW, dscale, dshift, scale, dres, dx_addend, dx_addend_mask, dx_mask, ws,
                      ws_bytes, false, hip_stream);
}

SOL_API int sol_block_bwd_noalloc(const sol_block_desc* desc, const void* dy, const void* x, const void* W, const void* y,
                          void* dx, float* dW, float* dscale, float* dshift, const float* scale, void* dres,
                          const void* dx_addend, const void* dx_addend_mask, const void* dx_mask, void* hip_stream) {
    return bwd_common(desc, dy, x, W, y, dx, dW, dscale, dshift, scale, dres, dx_addend, dx_addend_mask, dx_mask, nullptr,
                      (size_t)SOL_NOALLOC_SCRATCH_BYTES, true, hip_stream);
}

SOL_API size_t sol_block_bwd_noalloc_limit(void) { return (size_t)SOL_NOALLOC_SCRATCH_BYTES; }

SOL_API int sol_block_set_plan(const sol_block_desc* desc, int which, const sol_plan* plan) {
    if (!desc) return SOL_ERR_NULL;
    if (which != SOL_PLAN_FWD && which != SOL_PLAN_DGRAD && which != SOL_PLAN_WGRAD) return SOL_ERR_UNSUPPORTED;
    Geometry g;
    if (int e = check_desc(desc, &g)) return e;
    if (plan) {
        const bool stages_ok = plan->stages == 0 || (plan->stages >= 2 && plan->stages <= 4);
        if (!stages_ok || plan->tile < -1 || plan->tile > 4 || (plan->tile == 3 && plan->stages == 4) ||
            plan->splits < 0 || plan->splits > 65535)
            return SOL_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    if (plan) g_plans[plan_key(desc, which)] = *plan;
    else g_plans.erase(plan_key(desc, which));
    g_plan_count.store((int)g_plans.size(), std::memory_order_release);
    return SOL_OK;
}

SOL_API int sol_block_get_plan(const sol_block_desc* desc, int which, sol_plan* out) {
    if (!desc || !out) return SOL_ERR_NULL;
    if (which != SOL_PLAN_FWD && which != SOL_PLAN_DGRAD && which != SOL_PLAN_WGRAD) return SOL_ERR_UNSUPPORTED;
    *out = installed_plan(desc, which);
    return SOL_OK;
}

SOL_API void sol_reload_overrides(void) { load_knobs(); }

SOL_API void sol_clear_plans(void) {
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    g_plans.clear();
    g_plan_count.store(0, std::memory_order_release);
}

SOL_API int sol_l1_loss_grad(int32_t dtype, const void* y, const void* t, void* dy, int64_t numel, int32_t mask_by_y,
                             void* hip_stream) {
    if (dtype != SOL_F32 && dtype != SOL_BF16) return SOL_ERR_UNSUPPORTED;
    if (numel < 1) return SOL_ERR_SHAPE;
    if (!y || !t || !dy) return SOL_ERR_NULL;
    if (misaligned(y) || misaligned(t) || misaligned(dy)) return SOL_ERR_ALIGN;
    clear_stale_error();
    trace_point((hipStream_t)hip_stream, SOL_TRACE_L1_GRAD);
    const int st = launch_l1_grad(dtype, y, t, dy, numel, mask_by_y, (hipStream_t)hip_stream) == hipSuccess ? SOL_OK : SOL_ERR_LAUNCH;
    return st;
}

SOL_API int sol_maxpool_fwd(int32_t dtype, const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C, int32_t k,
                    int32_t stride, int32_t pad, void* hip_stream) {
    if (dtype != SOL_F32 && dtype != SOL_BF16) return SOL_ERR_UNSUPPORTED;
    if (N < 1 || H < 1 || W < 1 || C < 1 || k < 1 || stride < 1 || pad < 0 || pad >= k || H + 2 * pad < k ||
        W + 2 * pad < k)
        return SOL_ERR_SHAPE;
    if (!x || !y) return SOL_ERR_NULL;
    if (misaligned(x) || misaligned(y)) return SOL_ERR_ALIGN;
    clear_stale_error();
    trace_point((hipStream_t)hip_stream, SOL_TRACE_MAXPOOL);
    const int st = launch_maxpool(dtype, x, y, N, H, W, C, k, stride, pad, (hipStream_t)hip_stream) == hipSuccess
                       ? SOL_OK : SOL_ERR_LAUNCH;
    return st;
}

}  // extern "C"
