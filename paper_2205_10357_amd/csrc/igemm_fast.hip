// Pipelined variant of the implicit-GEMM kernel for the common case: source channels a
// multiple of 64 (every K slice of 64 lies inside one filter tap), output channels a multiple
// of 8, no ReLU mask on the gathered operand.
//
//  * operands go global -> LDS with asynchronous 16-byte copies (no register staging) into a
//    ring of NS stages; a slice is requested NS-1 iterations before it is multiplied, so HBM /
//    L2 latency is covered by several slices of MFMA work instead of one;
//  * the copies use buffer descriptors: the per-slice part of the address is a scalar, and padding
//    taps / rows past the end are given an out-of-range offset, which reads zeros;
//  * one raw workgroup barrier per slice, preceded by a vmcnt wait for exactly the slice that
//    is about to be read (a fenced barrier would drain the whole prefetch queue);
//  * the epilogue transposes the accumulators through LDS (fp32) so that every thread handles
//    8 consecutive channels of one pixel: residual / addend loads and output stores are 16-byte
//    pieces of contiguous NHWC rows, with a single rounding to bf16.
#include <type_traits>

#include "launch.h"
#include "reduce_rows.h"

namespace sol {

__device__ __forceinline__ int fast_swizzle(int row) { return (row + (row >> 3)) & 7; }

// Pins "NC async copies and NM MFMAs" as copy, MFMA, copy, MFMA, ...: a copy holds the wave's issue
// port for some twenty cycles, which one MFMA in flight covers and two copies in a row do not.
template <int NC, int NM>
__device__ __forceinline__ void fast_pin_copies_between_mfmas() {
    constexpr int PAIRS = NC < NM ? NC : NM;
#pragma unroll
    for (int c = 0; c < PAIRS; ++c) {
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    if constexpr (NC > PAIRS) __builtin_amdgcn_sched_group_barrier(0x010, NC - PAIRS, 0);
    if constexpr (NM > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, NM - PAIRS, 0);
}

template <int BP, int BC, int WP, int WC, int NS>
__global__ __launch_bounds__(256) void igemm_fast_kernel(const IgemmParams p) {
    static_assert(WP * WC == 4, "four waves per workgroup");
    constexpr int LP = BP / 32;            // async copies per thread and slice, pixel tile
    constexpr int LC = BC / 32;            // async copies per thread and slice, weight tile
    constexpr int LPS = LP + LC;
    constexpr int TP = BP / WP / 32;
    constexpr int TC = BC / WC / 32;
    constexpr int STAGE = (BP + BC) * 8;   // 16-byte chunks per stage
    constexpr int LDW = BC + 4;            // fp32 row pitch of the epilogue staging tile

    HIP_DYNAMIC_SHARED(uintx4, lds)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: keeps LDS bases scalar
    // all launch parameters in one batch of scalar loads; with one row class (forward, stride-1 data
    // gradient) the class is at a fixed place and belongs to the batch, else it costs a second round trip
    RowClass rc = p.cls[0];
    SOL_FETCH_NOW_8(p.src, p.wmat, p.out, p.scale, p.shift, p.addend, p.addend_mask, p.out_mask);
    SOL_FETCH_NOW_8(p.src_bytes, p.Hs, p.Ws, p.Cs, p.Nc, p.Hout, p.Wout, p.relu);
    SOL_FETCH_NOW_8(p.ncls, p.tiles_c, rc.rows, rc.Rh, rc.Rw, rc.h_mul, rc.h_off, rc.w_mul);
    SOL_FETCH_NOW_8(rc.w_off, rc.Th, rc.Tw, rc.tap_step, rc.oh_mul, rc.oh_off, rc.ow_mul, rc.ow_off);
    SOL_FETCH_NOW_8(rc.tile_begin, rc.linear, rc.b_off, rc.div_img.magic, rc.div_img.shift, rc.div_rw.magic,
                    rc.div_rw.shift, p.total_tiles);
    if ((int)blockIdx.x >= p.total_tiles) {    // workgroups behind the tiles: split reduction of the weight gradient
        // (the smaller tiles live on several workgroups per compute unit: the form that needs few registers)
        reduce_rows_riding<(BP * BC < 128 * 128)>(p.red, (int)blockIdx.x - p.total_tiles, p.red_blocks,
                                                  reinterpret_cast<float*>(lds));
        return;
    }
    const int bid = xcd_remap(blockIdx.x, p.total_tiles);     // total_tiles workgroups multiply
    const int tc = bid % p.tiles_c;
    int tp = bid / p.tiles_c;
    if (p.ncls > 1) {
        int cidx = 0;
#pragma unroll
        for (int i = 1; i < kMaxClasses; ++i)
            if (i < p.ncls && tp >= p.cls[i].tile_begin) cidx = i;
        rc = p.cls[cidx];
    }
    tp -= rc.tile_begin;
    const int row0 = tp * BP, ch0 = tc * BC;
    const int cpt = p.Cs >> 6;                         // slices per tap
    const int ntaps = rc.Th * rc.Tw;
    const int nk = ntaps * cpt;
    const long long K = (long long)ntaps * p.Cs;
    const int img_rows = rc.Rh * rc.Rw;
    const bf16_t* wmat = p.wmat + rc.b_off;

    // ---- epilogue role of this thread: 8 consecutive channels, rows pr0 + ps * RPP -------------
    constexpr int CPR = BC / 8;            // 8-channel chunks per tile row
    constexpr int RPP = 256 / CPR;         // tile rows per pass
    constexpr int PASSES = BP / RPP;
    const int cc = tid % CPR, pr0 = tid / CPR;
    const int ch = ch0 + cc * 8;
    const bool ch_ok = ch < p.Nc;
    floatx4 sc0 = {1.f, 1.f, 1.f, 1.f}, sc1 = sc0, sh0 = {0.f, 0.f, 0.f, 0.f}, sh1 = sh0;
    if (p.scale && ch_ok) {                // requested now, needed only after the main loop
        sc0 = *reinterpret_cast<const floatx4*>(p.scale + ch);
        sc1 = *reinterpret_cast<const floatx4*>(p.scale + ch + 4);
        sh0 = *reinterpret_cast<const floatx4*>(p.shift + ch);
        sh1 = *reinterpret_cast<const floatx4*>(p.shift + ch + 4);
    }

    // ---- what this thread copies: rows 32*i + 8*wave + (lane>>3), physical chunk lane&7 -------
    // Copies go through buffer descriptors: per row a loop-invariant vector offset, per slice one wave-uniform scalar
    // offset (tap and channel slice); a lane whose tap falls outside the image (or whose row does not exist) gets an
    // out-of-range vector offset and reads zeros.  The scalar offset must not be negative and the sum of the two
    // offsets must stay inside the descriptor for every valid (row, tap) -- the range check is on the sum.  Both hold
    // once the descriptor starts `margin` bytes before the tensor: margin = how far tap 0 of the first pixel lies
    // before the tensor (padding) plus how far the last tap lies before tap 0 (data gradient: taps walk backwards).
    // Only addresses inside the tensor are ever dereferenced.
    const int tap0_first = ((rc.h_off * p.Ws + rc.w_off) * p.Cs) * 2;
    const int tap_last = ((((rc.Th - 1) * p.Ws + (rc.Tw - 1)) * rc.tap_step) * p.Cs) * 2;
    const int delta_min = tap_last < 0 ? tap_last : 0;
    const unsigned margin = (unsigned)((tap0_first < 0 ? -tap0_first : 0) - delta_min);
    const buffer_rsrc_t src_rs = make_buffer_rsrc(reinterpret_cast<const char*>(p.src) - margin, p.src_bytes + margin);
    const buffer_rsrc_t w_rs = make_buffer_rsrc(wmat, (unsigned)(K * p.Nc * 2));
    const int j8 = lane >> 3, pc = lane & 7;
    // When the pixel rows need decoding (two divisions and the tap-validity mask per row), the weight copies of the
    // first NS-1 slices go out before it: their addresses are ready, and the decoding runs under their latency.  A
    // 1x1 / stride 1 source needs no decoding; there the copies go out slice by slice, pixels first (the pixel
    // operand is the one that comes from HBM).
    const bool weights_first = !(rc.linear & 1);
    unsigned wrowb[LC];
#pragma unroll
    for (int i = 0; i < LC; ++i) {
        const int lrow = 32 * i + 8 * wave + j8;
        const int c = ch0 + lrow;
        const int cl = pc ^ fast_swizzle(lrow);
        wrowb[i] = c < p.Nc ? (unsigned)(c * (int)K + cl * 8) * 2u : kOutOfRange;
    }
    auto weight_copies = [&](int stage, unsigned soff, int first, int last) {
#pragma unroll
        for (int iw = 0; iw < LC; ++iw)
            if (iw >= first && iw < last) dma16_buf_to_lds(w_rs, wrowb[iw], soff, lds + stage * STAGE + BP * 8 + (32 * iw + 8 * wave) * 8);
    };
    if (weights_first) {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < nk) weight_copies(s, (unsigned)(s * 128), 0, LC);
    }
    auto low_bits = [](int n) -> unsigned { return n >= 32 ? 0xffffffffu : (1u << n) - 1u; };   // n in 0 .. 32
    unsigned tap_rows = 0u;                // bit th * Tw set for every row of taps (at most 32 taps in all)
    for (int th = 0; th < rc.Th; ++th) tap_rows |= 1u << (th * rc.Tw);
    unsigned rowb[LP];                     // byte offset of (row, tap 0, logical chunk), modulo 2^32
    unsigned badtap[LP];                   // bit t set: tap t of this row lies outside the image
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const int lrow = 32 * i + 8 * wave + j8;
        const int r = row0 + lrow;
        const int cl = pc ^ fast_swizzle(lrow);        // logical chunk stored at physical chunk pc
        rowb[i] = 0u;
        badtap[i] = 0xffffffffu;
        if (r < rc.rows) {
            if (rc.linear & 1) {
                rowb[i] = (unsigned)(r * p.Cs + cl * 8) * 2u;
                badtap[i] = 0xfffffffeu;
            } else {
                const int n = (int)fast_div((uint32_t)r, rc.div_img), rem = r - n * img_rows;
                const int rh = (int)fast_div((uint32_t)rem, rc.div_rw), rw = rem - rh * rc.Rw;
                const int h0 = rh * rc.h_mul + rc.h_off, w0 = rw * rc.w_mul + rc.w_off;
                rowb[i] = (unsigned)(((n * p.Hs + h0) * p.Ws + w0) * p.Cs + cl * 8) * 2u;
                // Taps th with 0 <= h0 + th * tap_step < Hs form one interval [hl, hh] (tap_step = +1 or -1), likewise
                // [wl, wh] along the width.  Tap (th, tw) is bit th * Tw + tw: the valid taps are the width interval
                // repeated in every row of taps (one multiplication by the bit pattern 1, 1 << Tw, 1 << 2 Tw, ...),
                // cut down to the rows hl .. hh.
                auto interval = [&](int v0, int extent, int taps, int& l, int& h) {
                    const int lo = rc.tap_step > 0 ? -v0 : v0 - extent + 1;
                    const int hi = rc.tap_step > 0 ? extent - 1 - v0 : v0;
                    l = lo > 0 ? lo : 0;
                    h = hi < taps - 1 ? hi : taps - 1;
                };
                int hl, hh, wl, wh;
                interval(h0, p.Hs, rc.Th, hl, hh);
                interval(w0, p.Ws, rc.Tw, wl, wh);
                unsigned good = 0u;
                if (hh >= hl && wh >= wl) {
                    const unsigned wgood = low_bits(wh + 1) & ~low_bits(wl);
                    good = (wgood * tap_rows) & low_bits((hh + 1) * rc.Tw) & ~low_bits(hl * rc.Tw);
                }
                badtap[i] = ~good;
            }
        }
    }
    // Requests are issued slice by slice in ring order; a slice is requested in parts so that the copies can be issued
    // between the MFMAs of the slice being multiplied.  Everything a request needs is ready before it starts: the
    // scalar offsets of the next slice (pixel and weight operand) and, after a change of tap, the vector offsets are
    // computed right after the last copy of the previous request, under the MFMAs -- not between the barrier and the
    // first copy, where the whole wave would wait for a chain of dependent scalar instructions.  Within a tap a slice
    // costs two scalar adds.
    int q_cs = 0, q_th = 0, q_tw = 0, q_tap = 0, q_stage = 0;
    unsigned s_pix = (unsigned)(-delta_min);   // scalar offset of the pixel copies: tap + channel slice, biased to be >= 0
    unsigned s_w = 0u;                         // scalar offset of the weight copies: 128 bytes per slice
    unsigned voff[LP];                         // vector offset of this thread's pixel copies for the current tap:
#pragma unroll                                 // all-ones where the tap lies outside the image
    for (int i = 0; i < LP; ++i) voff[i] = (rowb[i] + margin + (unsigned)delta_min) | (unsigned)__builtin_amdgcn_sbfe((int)badtap[i], 0, 1);
    auto next_pixel_slice = [&]() {
        if (__builtin_expect(++q_cs == cpt, 0)) {      // next tap (never taken again by a 1x1 layer)
            q_cs = 0;
            ++q_tap;
            if (++q_tw == rc.Tw) {
                q_tw = 0;
                ++q_th;
            }
            s_pix = (unsigned)((((q_th * p.Ws + q_tw) * rc.tap_step) * p.Cs) * 2 - delta_min);
#pragma unroll
            for (int i = 0; i < LP; ++i)
                voff[i] = (rowb[i] + margin + (unsigned)delta_min) | (unsigned)__builtin_amdgcn_sbfe((int)badtap[i], q_tap & 31, 1);
        } else {
            s_pix += 128u;
        }
    };
    auto request_part = [&](int stage, int part, int nparts) {
        uintx4* st = lds + stage * STAGE;
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            if (i < (part * LPS) / nparts || i >= ((part + 1) * LPS) / nparts) continue;
            if (i < LP) dma16_buf_to_lds(src_rs, voff[i], s_pix, st + (32 * i + 8 * wave) * 8);
            else weight_copies(stage, s_w, i - LP, i - LP + 1);
        }
        if (part == nparts - 1) {
            s_w += 128u;
            next_pixel_slice();
        }
    };
    // for the loops that do not know the ring stage at compile time
    auto request_part_rt = [&](int part, int nparts) {
        request_part(q_stage, part, nparts);
        if (part == nparts - 1) q_stage = q_stage + 1 == NS ? 0 : q_stage + 1;
    };

    const int wp = wave % WP, wc = wave / WP;
    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // pixel copies of the first NS-1 slices (with weights_first their weight copies are on their way already)
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) {
#pragma unroll
            for (int i = 0; i < LP; ++i) dma16_buf_to_lds(src_rs, voff[i], s_pix, lds + s * STAGE + (32 * i + 8 * wave) * 8);
            if (!weights_first) weight_copies(s, s_w, 0, LC);
            next_pixel_slice();
            s_w += 128u;
            q_stage = q_stage + 1 == NS ? 0 : q_stage + 1;
        }

    // LDS chunk index (inside a stage) of this lane's operand fragment for each of the 4 steps
    int wfo[TC][4], pfo[TP][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int chunk = 2 * ks + (lane >> 5);
#pragma unroll
        for (int i = 0; i < TC; ++i) {
            const int r = wc * (BC / WC) + i * 32 + (lane & 31);
            wfo[i][ks] = BP * 8 + r * 8 + (chunk ^ fast_swizzle(r));
        }
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int r = wp * (BP / WP) + j * 32 + (lane & 31);
            pfo[j][ks] = r * 8 + (chunk ^ fast_swizzle(r));
        }
    }

    bf16x8 wf[2][TC], pf[2][TP];           // operand fragments of two consecutive steps
    auto read_frags = [&](int buf, const uintx4* st, int ks) {
#pragma unroll
        for (int i = 0; i < TC; ++i) wf[buf][i] = __builtin_bit_cast(bf16x8, st[wfo[i][ks]]);
#pragma unroll
        for (int j = 0; j < TP; ++j) pf[buf][j] = __builtin_bit_cast(bf16x8, st[pfo[j][ks]]);
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], pf[buf][j], acc[i][j], 0, 0, 0);
    };

    if constexpr (NS >= 3) {
        // Slices overlap: the fragments of a slice's first step are read during the last step of the
        // slice before it, so the matrix pipe never waits for LDS latency at a slice boundary.  The one
        // barrier per slice sits in the middle of slice kt (after its step 0 is issued) and does two jobs:
        // slice kt+1 has landed for every wave (each waited for its own copies first), and no wave reads
        // slice kt-1 any more, so its stage may be overwritten by the copies of slice kt+NS-1, which are
        // issued after the barrier in three parts between the MFMA groups.  The instruction order
        // "fragments of the next step, copies, MFMAs of this step" is pinned with scheduling-group
        // barriers: left alone, the scheduler sinks the LDS reads below the MFMAs that precede their use.
        // The ring stage of a slice is a compile-time constant (the loop below advances NS slices per iteration), so the
        // stage's base is an immediate of the fragment reads instead of a vector add per read: with one wave per SIMD
        // the in-order issue of that wave is what bounds the loop, and the ~16 address adds per slice were ~9 % of it.
        // (Stages beyond the 64 KB reach of the immediate cost one hoisted address register per fragment; the
        // 256 x 128 tile has none to spare and keeps the stage in a register.)
        auto slice = [&](auto stage, auto next_tag, auto more_tag) {
            const int S = stage;                               // slice kt lives in ring stage S = kt % NS
            constexpr bool NEXT = decltype(next_tag)::value;   // slice kt+1 exists
            constexpr bool MORE = decltype(more_tag)::value;   // slice kt+NS-1 exists and is requested here
            const uintx4* st = lds + S * STAGE;
            const uintx4* stn = lds + ((S + 1) % NS) * STAGE;
            auto request = [&](int part) {                     // slice kt+NS-1 goes where slice kt-1 was
                if constexpr (std::is_same_v<decltype(stage), int>) request_part_rt(part, 3);
                else request_part((S + NS - 1) % NS, part, 3);
            };
            read_frags(1, st, 1);
            multiply(0);
            __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, TC * TP, 0);
            read_frags(0, st, 2);
            __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
            if constexpr (NEXT) {
                // copies of slices kt+2 .. kt+NS-2 may stay in flight (none once requests have stopped)
                __builtin_amdgcn_s_waitcnt(MORE ? (0x0f70 | (((NS - 3) * LPS) & 15) | ((((NS - 3) * LPS) >> 4) << 14))
                                                : 0x0f70);
                wg_barrier();
            }
            if constexpr (MORE) request(0);
            multiply(1);
            fast_pin_copies_between_mfmas<MORE ? LPS / 3 : 0, TC * TP>();
            read_frags(1, st, 3);
            if constexpr (MORE) request(1);
            multiply(0);
            __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
            fast_pin_copies_between_mfmas<MORE ? (2 * LPS) / 3 - LPS / 3 : 0, TC * TP>();
            if constexpr (NEXT) read_frags(0, stn, 0);
            if constexpr (MORE) request(2);
            multiply(1);
            if constexpr (NEXT) __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
            fast_pin_copies_between_mfmas<MORE ? LPS - (2 * LPS) / 3 : 0, TC * TP>();
        };

        // Slice 0 must have landed.  Requested slice by slice, slices 1 .. NS-2 may still be in flight.  Requested
        // weights first, only the pixel copies of slice NS-2 were issued behind those of slice NS-3: that wait lets
        // slices 0 .. NS-3 land (the in-loop waits count whole slices, which holds from slice NS-2 on).
        if (nk < NS - 1) wait_vm_and_lds<0>();
        else if (weights_first) wait_vm_and_lds<LP>();
        else wait_vm_and_lds<(NS - 2) * LPS>();
        wg_barrier();
        if (nk > 0) {                // a row class without taps (strided data gradient) has nothing to multiply
            read_frags(0, lds, 0);
            // R slices starting at a multiple of NS, written out: slice I sits in stage I % NS, has a successor
            // unless it is the last, and requests slice I + NS - 1 if that exists
            auto run = [&](auto r_tag, auto all_tag) {
                constexpr int R = decltype(r_tag)::value;
                constexpr bool ALL = decltype(all_tag)::value;     // a full group in the middle: every slice requests
                auto one = [&](auto i_tag) {
                    constexpr int I = decltype(i_tag)::value;
                    if constexpr (I < R)
                        slice(std::integral_constant<int, I % NS>{}, std::integral_constant<bool, ALL || (I < R - 1)>{},
                              std::integral_constant<bool, ALL || (I + NS - 1 < R)>{});
                };
                one(std::integral_constant<int, 0>{});
                one(std::integral_constant<int, 1>{});
                one(std::integral_constant<int, 2>{});
                one(std::integral_constant<int, 3>{});
                one(std::integral_constant<int, 4>{});
                one(std::integral_constant<int, 5>{});
            };
            static_assert(2 * NS - 2 <= 6, "the tail is written out for at most six slices");
            int kt = 0;
            if constexpr (BP * BC > 128 * 128) {
                for (; kt + NS - 1 < nk; ++kt) slice(kt % NS, std::true_type{}, std::true_type{});
                for (; kt + 1 < nk; ++kt) slice(kt % NS, std::true_type{}, std::false_type{});
                slice(kt % NS, std::false_type{}, std::false_type{});
            } else {
                for (; kt + 2 * NS - 2 < nk; kt += NS) run(std::integral_constant<int, NS>{}, std::true_type{});
                switch (nk - kt) {           // 1 .. 2*NS - 2 slices are left
                    case 1: run(std::integral_constant<int, 1>{}, std::false_type{}); break;
                    case 2: run(std::integral_constant<int, 2>{}, std::false_type{}); break;
                    case 3: run(std::integral_constant<int, 3>{}, std::false_type{}); break;
                    case 4: run(std::integral_constant<int, 4>{}, std::false_type{}); break;
                    case 5: if constexpr (NS >= 4) run(std::integral_constant<int, 5>{}, std::false_type{}); break;
                    default: if constexpr (NS >= 4) run(std::integral_constant<int, 6>{}, std::false_type{}); break;
                }
            }
        }
    } else {
        // Two stages: one K slice = wait for it, multiply it, and (MORE) request the next one in four
        // parts between the MFMA groups; one barrier at the start of every slice.
        auto slice = [&](int kt, auto more_tag) {
            constexpr bool MORE = decltype(more_tag)::value;
            const uintx4* st = lds + (kt % NS) * STAGE;
            read_frags(0, st, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks < 3) read_frags(nxt, st, ks + 1);
                if constexpr (MORE) request_part_rt(ks, 4);
                multiply(cur);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);            // fragments of step 0
#define SOL_SGB_STEP(KS)                                                                              \
            if constexpr ((KS) < 3) __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);              \
            fast_pin_copies_between_mfmas<MORE ? (((KS) + 1) * LPS) / 4 - ((KS) * LPS) / 4 : 0, TC * TP>();
            SOL_SGB_STEP(0)
            SOL_SGB_STEP(1)
            SOL_SGB_STEP(2)
            SOL_SGB_STEP(3)
#undef SOL_SGB_STEP
        };

        int kt = 0;
        for (; kt + NS - 1 < nk; ++kt) {
            wait_vm_and_lds<(NS - 2) * LPS>();   // slice kt must have landed
            wg_barrier();            // every wave's part of slice kt is in LDS; slice kt-1 is no longer read
            slice(kt, std::true_type{});
        }
        for (; kt < nk; ++kt) {
            wait_vm_and_lds<0>();
            wg_barrier();
            slice(kt, std::false_type{});
        }
    }

    // ---- epilogue: accumulators -> LDS [pixel][channel] fp32 -> 8 channels per thread --------
    float* stg = reinterpret_cast<float*>(lds);
    // output offsets of this thread's rows, and its addend pieces (requested before the barriers)
    long long oofs[PASSES];
    bool ovalid[PASSES];
    uintx4 addv[PASSES], addm[PASSES], outm[PASSES];
    if (rc.linear & 2) {                 // output pixel index == row: offsets advance by a constant
        const long long o0 = (long long)(row0 + pr0) * p.Nc + ch;
        const long long ostep = (long long)RPP * p.Nc;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            ovalid[ps] = ch_ok && (row0 + pr0 + ps * RPP) < rc.rows;
            oofs[ps] = o0 + ps * ostep;
        }
    } else {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = row0 + pr0 + ps * RPP;
            ovalid[ps] = ch_ok && r < rc.rows;
            const int rr = ovalid[ps] ? r : 0;
            const int n = (int)fast_div((uint32_t)rr, rc.div_img), rem = rr - n * img_rows;
            const int rh = (int)fast_div((uint32_t)rem, rc.div_rw), rw = rem - rh * rc.Rw;
            const long long opix = ((long long)n * p.Hout + (rh * rc.oh_mul + rc.oh_off)) * p.Wout +
                                   (rw * rc.ow_mul + rc.ow_off);
            oofs[ps] = opix * p.Nc + ch;
        }
    }
    const uintx4 kOnes = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        addv[ps] = uintx4{0u, 0u, 0u, 0u};
        addm[ps] = kOnes;
        outm[ps] = kOnes;
    }
    if (p.addend) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
            if (ovalid[ps]) addv[ps] = *reinterpret_cast<const uintx4*>(p.addend + oofs[ps]);
        if (p.addend_mask) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                if (ovalid[ps]) addm[ps] = *reinterpret_cast<const uintx4*>(p.addend_mask + oofs[ps]);
        }
    }
    if (p.out_mask) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
            if (ovalid[ps]) outm[ps] = *reinterpret_cast<const uintx4*>(p.out_mask + oofs[ps]);
    }
    wait_vm_and_lds<PASSES * 3 < 64 ? PASSES * 3 : 63>();   // LDS reads done; the epilogue loads may stay in flight
    wg_barrier();                                   // all operand reads done, LDS can be reused
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int pr = wp * (BP / WP) + j * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = wc * (BC / WC) + i * 32 + 8 * q + 4 * (lane >> 5);
                *reinterpret_cast<floatx4*>(stg + pr * LDW + c) =
                    floatx4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            }
    }
    wait_vm_and_lds<PASSES * 3 < 64 ? PASSES * 3 : 63>();
    wg_barrier();

    // all staged rows first (independent LDS reads), then the arithmetic, then the stores
    floatx4 va[PASSES], vb[PASSES];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int pr = pr0 + ps * RPP;
        va[ps] = *reinterpret_cast<const floatx4*>(stg + pr * LDW + cc * 8);
        vb[ps] = *reinterpret_cast<const floatx4*>(stg + pr * LDW + cc * 8 + 4);
    }
    const bool has_addend = p.addend != nullptr, has_outmask = p.out_mask != nullptr, relu = p.relu != 0;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        float v[8] = {va[ps][0], va[ps][1], va[ps][2], va[ps][3], vb[ps][0], vb[ps][1], vb[ps][2], vb[ps][3]};
#pragma unroll
        for (int e = 0; e < 4; ++e) {        // identity (1, 0) when the launch has no affine
            v[e] = fmaf(sc0[e], v[e], sh0[e]);
            v[e + 4] = fmaf(sc1[e], v[e + 4], sh1[e]);
        }
        if (has_addend) {
            const uintx4 a = mask_where_positive(addv[ps], addm[ps]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[2 * e] += __uint_as_float(a[e] << 16);
                v[2 * e + 1] += __uint_as_float(a[e] & 0xffff0000u);
            }
        }
        if (relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;   // never -0, NaN -> 0
        }
        uintx4 out = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                      pack_bf16x2(v[6], v[7])};
        if (has_outmask) out = mask_where_positive(out, outm[ps]);
        if (ovalid[ps]) store16_through(p.out + oofs[ps], out);
    }
}

template <int BP, int BC, int WP, int WC, int NS>
static hipError_t launch_fast_tile(const IgemmParams& p, hipStream_t stream) {
    const size_t stages = (size_t)NS * (BP + BC) * 8 * 16;
    const size_t epi = (size_t)BP * (BC + 4) * 4;
    const size_t smem = stages > epi ? stages : epi;
    auto kern = igemm_fast_kernel<BP, BC, WP, WC, NS>;
    static std::atomic<size_t> granted{0};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, granted); e != hipSuccess) return e;
    SOL_LAUNCH(kern, dim3(p.total_tiles + p.red_blocks), dim3(256), smem, stream, p);
    return hipGetLastError();
}

// tile: 0 = 128 x 128, 1 = 128 pixels x 64 channels, 2 = 64 x 64, 3 = 256 x 128; stages: 2, 3 or 4
hipError_t launch_igemm_fast(const IgemmParams& p, int tile, int stages, hipStream_t stream) {
    if (p.total_tiles <= 0) return hipSuccess;
    switch (tile * 8 + stages) {
        case 0 * 8 + 2: return launch_fast_tile<128, 128, 2, 2, 2>(p, stream);
        case 0 * 8 + 3: return launch_fast_tile<128, 128, 2, 2, 3>(p, stream);
        case 0 * 8 + 4: return launch_fast_tile<128, 128, 2, 2, 4>(p, stream);
        case 1 * 8 + 2: return launch_fast_tile<128, 64, 2, 2, 2>(p, stream);
        case 1 * 8 + 3: return launch_fast_tile<128, 64, 2, 2, 3>(p, stream);
        case 1 * 8 + 4: return launch_fast_tile<128, 64, 2, 2, 4>(p, stream);
        case 2 * 8 + 2: return launch_fast_tile<64, 64, 2, 2, 2>(p, stream);
        case 2 * 8 + 3: return launch_fast_tile<64, 64, 2, 2, 3>(p, stream);
        case 2 * 8 + 4: return launch_fast_tile<64, 64, 2, 2, 4>(p, stream);
        case 3 * 8 + 2: return launch_fast_tile<256, 128, 2, 2, 2>(p, stream);
        case 3 * 8 + 3: return launch_fast_tile<256, 128, 2, 2, 3>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

void igemm_fast_tile_shape(int tile, int* bp, int* bc) {
    static const int shapes[4][2] = {{128, 128}, {128, 64}, {64, 64}, {256, 128}};
    const int t = (tile < 0 || tile > 3) ? 2 : tile;
    *bp = shapes[t][0];
    *bc = shapes[t][1];
}

}  // namespace sol
