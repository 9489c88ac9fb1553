// "Panel" variant of the pipelined implicit-GEMM kernel for 1x1 / stride-1 launches with a short reduction and a
// wide output (the expand layer of a bottleneck, forward, and the data gradient of its reduce layer): source
// channels 64, 128 or 256, output channels a multiple of 128.
//
// Such a launch is bound by memory and by per-workgroup latency, not by the matrix cores: with one output tile per
// workgroup every tile pays its own start-up (arguments, first copies from HBM) and its own epilogue, and the pixel
// operand is copied into LDS once per channel tile.  Here a workgroup keeps its 128-pixel panel of the source in
// LDS (all K slices, copied once) and walks over several 128-channel tiles of the output: the weight slices of the
// tiles stream through a ring of four stages without a break at tile boundaries, and the epilogue operands of the
// next tile are requested one tile ahead, so start-up is paid once per workgroup and the copies of tile t+1 are in
// flight (or have landed) while tile t is finished.
//
//  * LDS: NK pixel slices (16 KiB each) + 4 weight slices (16 KiB each) + scale / shift of the workgroup's
//    channels (8 KiB); slice layout, swizzle, fragment reads and MFMA order are those of the 128 x 128 tile of
//    igemm_fast_kernel, so every output element is accumulated in the same order and the results are identical
//    bit for bit.
//  * The epilogue works from the accumulators without an LDS transpose: a 32 x 32 MFMA result leaves a lane with
//    4 consecutive channels of one pixel per group of 8; exchanging registers between lanes l and l+32
//    (v_permlane32_swap) gives every lane 8 consecutive channels, i.e. the 16-byte pieces of NHWC rows that the
//    addend loads and the stores work on.  No barrier is needed and the weight ring stays live.
//  * vmcnt bookkeeping: loads complete in order, so "slice j+1 has landed" is "at most N loads issued after its
//    last copy are outstanding".  N is a compile-time constant per position in the tile: one more weight slice,
//    plus the epilogue loads of the next tile where a tile boundary lies in between.  Stores only make a wait
//    stricter.  Once requests have stopped (last three slices of a workgroup) the waits are for everything.
#include <type_traits>

#include "launch.h"
#include "reduce_rows.h"

namespace sol {

__device__ __forceinline__ int panel_swizzle(int row) { return (row + (row >> 3)) & 7; }

constexpr int kPanelMaxTiles = 8;          // channel tiles per workgroup (size of the scale / shift cache)

template <int NC, int NM>
__device__ __forceinline__ void panel_pin_copies_between_mfmas() {
    constexpr int PAIRS = NC < NM ? NC : NM;
#pragma unroll
    for (int c = 0; c < PAIRS; ++c) {
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    if constexpr (NC > PAIRS) __builtin_amdgcn_sched_group_barrier(0x010, NC - PAIRS, 0);
    if constexpr (NM > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, NM - PAIRS, 0);
}

template <int NK, bool HAS_OMASK>
__global__ __launch_bounds__(256) void igemm_panel_kernel(const IgemmParams p) {
    constexpr int NSW = 4;                 // weight ring
    constexpr int LP = 4, LC = 4;          // copies per thread and slice, pixel / weight operand
    constexpr int STAGE = 128 * 8;         // 16-byte chunks per operand slice (128 rows x 128 bytes)
    constexpr int TP = 2, TC = 2;          // 32 x 32 MFMA tiles per wave and direction
    constexpr int R = 8 + (HAS_OMASK ? 8 : 0);   // epilogue loads per thread and tile

    HIP_DYNAMIC_SHARED(uintx4, lds)
    uintx4* const ldsA = lds;
    uintx4* const ldsW = lds + NK * STAGE;
    float* const aff = reinterpret_cast<float*>(lds + (NK + NSW) * STAGE);   // [0, 1024): scale, [1024, 2048): shift

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const RowClass& rc = p.cls[0];
    SOL_FETCH_NOW_8(p.src, p.wmat, p.out, p.scale, p.shift, p.addend, p.out_mask, p.src_bytes);
    SOL_FETCH_NOW_8(p.Cs, p.Nc, p.relu, p.tiles_c, p.total_tiles, p.panel_groups, p.panel_tiles, rc.rows);

    if ((int)blockIdx.x >= p.total_tiles) {    // workgroups behind the panels: split reduction of the weight gradient
        reduce_rows_riding<false>(p.red, (int)blockIdx.x - p.total_tiles, p.red_blocks, reinterpret_cast<float*>(lds));
        return;
    }
    const int bid = xcd_remap(blockIdx.x, p.total_tiles);
    // (the quotient is computed in vector registers; without the broadcast everything derived from it, the weight
    // descriptor included, would count as lane-dependent)
    const int panel = __builtin_amdgcn_readfirstlane(bid / p.panel_groups), grp = bid - panel * p.panel_groups;
    const int row0 = panel * 128;
    const int t_begin = grp * p.panel_tiles;
    const int t_count = min(p.panel_tiles, p.tiles_c - t_begin);
    const int ch_begin = t_begin * 128;
    const int K = p.Cs;                                    // = 64 * NK
    const int J = t_count * NK;                            // weight slices of this workgroup

    // ---- scale / shift of this workgroup's channels -> LDS (loads now, LDS writes after the copies are issued)
    float sv[kPanelMaxTiles * 128 / 256], hv[kPanelMaxTiles * 128 / 256];
#pragma unroll
    for (int u = 0; u < kPanelMaxTiles * 128 / 256; ++u) {
        const int c = u * 256 + tid;
        sv[u] = 1.f;
        hv[u] = 0.f;
        if (p.scale && c < t_count * 128) {
            sv[u] = p.scale[ch_begin + c];
            hv[u] = p.shift[ch_begin + c];
        }
    }

    // ---- copy role (as in igemm_fast_kernel): rows 32*i + 8*wave + (lane>>3), physical chunk lane&7
    const buffer_rsrc_t src_rs = make_buffer_rsrc(p.src, p.src_bytes);
    // (32-bit scalar arithmetic for the byte offset: a 64-bit product would be formed in vector registers and the
    // descriptor would have to be re-broadcast at every copy)
    const unsigned w_first = (unsigned)ch_begin * (unsigned)K * 2u;
    // the descriptor spans every tile of this workgroup: the range check takes the scalar offset into account
    const buffer_rsrc_t w_rs = make_buffer_rsrc(reinterpret_cast<const char*>(p.wmat) + w_first, (unsigned)(t_count * 128 * K * 2));
    const int j8 = lane >> 3, pc = lane & 7;
    unsigned arow[LP], wrow[LC];
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const int lrow = 32 * i + 8 * wave + j8;
        const int cl = pc ^ panel_swizzle(lrow);
        const int r = row0 + lrow;
        arow[i] = r < rc.rows ? (unsigned)(r * p.Cs + cl * 8) * 2u : kOutOfRange;
        wrow[i] = (unsigned)(lrow * K + cl * 8) * 2u;
    }
#pragma unroll
    for (int s = 0; s < NK; ++s)
#pragma unroll
        for (int i = 0; i < LP; ++i) dma16_buf_to_lds(src_rs, arow[i], (unsigned)(s * 128), ldsA + s * STAGE + (32 * i + 8 * wave) * 8);

    // weight slices are requested in stream order j = tile * NK + slice; the scalar offset walks along the K-contiguous
    // rows inside a tile (128 bytes per slice) and jumps to the next 128 rows at a tile boundary
    int q_s = 0, q_stage = 0;
    unsigned q_soff = 0u;
    auto request_w = [&](int first, int last) {
#pragma unroll
        for (int iw = 0; iw < LC; ++iw)
            if (iw >= first && iw < last) dma16_buf_to_lds(w_rs, wrow[iw], q_soff, ldsW + q_stage * STAGE + (32 * iw + 8 * wave) * 8);
        if (last == LC) {
            q_stage = (q_stage + 1) & (NSW - 1);
            q_soff += 128u;
            if (++q_s == NK) {
                q_s = 0;
                q_soff += (unsigned)(127 * K * 2);
            }
        }
    };
#pragma unroll
    for (int jj = 0; jj < NSW - 1; ++jj)
        if (jj < J) request_w(0, LC);

    // ---- MFMA / epilogue role: wave grid 2 (pixels) x 2 (channels), 64 x 64 each
    const int wp = wave & 1, wc = wave >> 1;
    const int h = lane >> 5;
    // after the lane exchange this lane owns, per (pixel tile j, channel tile i, pair qp), 8 consecutive channels
    // wc*64 + i*32 + qp*16 + h*8 .. +7 of pixel row0 + wp*64 + j*32 + (lane & 31)
    const buffer_rsrc_t out_rs = make_buffer_rsrc(p.out, (unsigned)((long long)rc.rows * p.Nc * 2));
    const buffer_rsrc_t add_rs = make_buffer_rsrc(p.addend ? p.addend : p.out, p.addend ? (unsigned)((long long)rc.rows * p.Nc * 2) : 0u);
    const buffer_rsrc_t om_rs = make_buffer_rsrc(p.out_mask ? p.out_mask : p.out, p.out_mask ? (unsigned)((long long)rc.rows * p.Nc * 2) : 0u);
    unsigned eoff[TP][TC][2];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int r = row0 + wp * 64 + j * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp)
                eoff[j][i][qp] = r < rc.rows ? (unsigned)(((long long)r * p.Nc + ch_begin + wc * 64 + i * 32 + qp * 16 + h * 8) * 2) : kOutOfRange;
    }
    uintx4 addv[TP][TC][2], outm[TP][TC][2];
    auto request_epilogue_operands = [&](int ti) {
        asm volatile("" ::: "memory");          // keeps these loads at this place of the load stream
        const unsigned soff = (unsigned)(ti * 256);
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int i = 0; i < TC; ++i)
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    addv[j][i][qp] = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(add_rs, eoff[j][i][qp], soff, 0));
                    if constexpr (HAS_OMASK)
                        outm[j][i][qp] = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(om_rs, eoff[j][i][qp], soff, 0));
                }
        asm volatile("" ::: "memory");
    };
    request_epilogue_operands(0);

#pragma unroll
    for (int u = 0; u < kPanelMaxTiles * 128 / 256; ++u) {
        aff[u * 256 + tid] = sv[u];
        aff[1024 + u * 256 + tid] = hv[u];
    }

    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // LDS chunk index (inside a slice) of this lane's operand fragment for each of the 4 steps
    int wfo[TC][4], pfo[TP][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int chunk = 2 * ks + (lane >> 5);
#pragma unroll
        for (int i = 0; i < TC; ++i) {
            const int r = wc * 64 + i * 32 + (lane & 31);
            wfo[i][ks] = r * 8 + (chunk ^ panel_swizzle(r));
        }
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int r = wp * 64 + j * 32 + (lane & 31);
            pfo[j][ks] = r * 8 + (chunk ^ panel_swizzle(r));
        }
    }
    bf16x8 wf[2][TC], pf[2][TP];
    auto read_frags = [&](int buf, const uintx4* sa, const uintx4* sw, int ks) {
#pragma unroll
        for (int i = 0; i < TC; ++i) wf[buf][i] = __builtin_bit_cast(bf16x8, sw[wfo[i][ks]]);
#pragma unroll
        for (int j = 0; j < TP; ++j) pf[buf][j] = __builtin_bit_cast(bf16x8, sa[pfo[j][ks]]);
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], pf[buf][j], acc[i][j], 0, 0, 0);
    };

    // One slice (stream position jpos, slice S of its tile).  FULL: the slice three ahead exists and is requested here,
    // waits are exact.  Otherwise nothing is requested any more and the wait is for everything.
    int jpos = 0;
    auto slice = [&](auto s_tag, auto full_tag) {
        constexpr int S = decltype(s_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;
        // loads issued behind the last copy of slice jpos+1 when this slice waits for it: the copies of slice jpos+2 and
        // the epilogue loads of every tile boundary that lies one or two slices back
        constexpr int BOUNDARIES = ((((S - 1) % NK + NK) % NK) == NK - 1 ? 1 : 0) + ((((S - 2) % NK + NK) % NK) == NK - 1 ? 1 : 0);
        constexpr int N_WAIT = LC + R * BOUNDARIES;
        static_assert(N_WAIT < 64, "vmcnt is a 6-bit field");
        const bool has_next = jpos + 1 < J;
        const uintx4* sa = ldsA + S * STAGE;
        const uintx4* sw = ldsW + (jpos & (NSW - 1)) * STAGE;
        read_frags(1, sa, sw, 1);
        multiply(0);
        __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, TC * TP, 0);
        read_frags(0, sa, sw, 2);
        __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
        if (FULL || has_next) {
            // (with one slice per tile, the very first slice has only one tile boundary -- the start -- behind it)
            constexpr int N_FIRST = LC + R * (BOUNDARIES > 1 ? 1 : BOUNDARIES);
            if (!FULL) __builtin_amdgcn_s_waitcnt(0x0f70);
            else if (N_FIRST != N_WAIT && jpos == 0) __builtin_amdgcn_s_waitcnt(0x0f70 | (N_FIRST & 15) | ((N_FIRST >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0f70 | (N_WAIT & 15) | ((N_WAIT >> 4) << 14));
            wg_barrier();
        }
        if constexpr (FULL) request_w(0, 1);
        multiply(1);
        panel_pin_copies_between_mfmas<FULL ? 1 : 0, TC * TP>();
        read_frags(1, sa, sw, 3);
        if constexpr (FULL) request_w(1, 2);
        multiply(0);
        __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
        panel_pin_copies_between_mfmas<FULL ? 1 : 0, TC * TP>();
        if (FULL || has_next) read_frags(0, ldsA + ((S + 1) % NK) * STAGE, ldsW + ((jpos + 1) & (NSW - 1)) * STAGE, 0);
        if constexpr (FULL) request_w(2, LC);
        multiply(1);
        if constexpr (FULL) __builtin_amdgcn_sched_group_barrier(0x100, TC + TP, 0);
        panel_pin_copies_between_mfmas<FULL ? 2 : 0, TC * TP>();
        ++jpos;
    };

    const bool relu = p.relu != 0, has_addend = p.addend != nullptr;
    auto epilogue = [&](int ti) {
        const unsigned soff = (unsigned)(ti * 256);
        const float* sc = aff + ti * 128 + wc * 64 + h * 8;
        const float* sh = sc + 1024;
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                const floatx4 s0 = *reinterpret_cast<const floatx4*>(sc + i * 32 + qp * 16);
                const floatx4 s1 = *reinterpret_cast<const floatx4*>(sc + i * 32 + qp * 16 + 4);
                const floatx4 b0 = *reinterpret_cast<const floatx4*>(sh + i * 32 + qp * 16);
                const floatx4 b1 = *reinterpret_cast<const floatx4*>(sh + i * 32 + qp * 16 + 4);
#pragma unroll
                for (int j = 0; j < TP; ++j) {
                    float v[8];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // X: group 2*qp, Y: group 2*qp+1 of the MFMA result; lanes 32..63 of X trade places with lanes 0..31 of Y
                        const auto sw2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][8 * qp + r]),
                                                                          __float_as_uint(acc[i][j][8 * qp + 4 + r]), false, false);
                        v[r] = __uint_as_float(sw2[0]);
                        v[4 + r] = __uint_as_float(sw2[1]);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = fmaf(s0[e], v[e], b0[e]);
                        v[e + 4] = fmaf(s1[e], v[e + 4], b1[e]);
                    }
                    if (has_addend) {
                        const uintx4 a = addv[j][i][qp];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v[2 * e] += __uint_as_float(a[e] << 16);
                            v[2 * e + 1] += __uint_as_float(a[e] & 0xffff0000u);
                        }
                    }
                    if (relu) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    uintx4 out = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                    if constexpr (HAS_OMASK) out = mask_where_positive(out, outm[j][i][qp]);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned, out),
                                                           out_rs, eoff[j][i][qp], soff, 0);
                }
            }
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    };

    // slice 0 and the pixel panel must have landed; behind the last copy of slice 0 came slices 1, 2 and the epilogue loads of tile 0
    if (J >= NSW - 1) wait_vm_and_lds<2 * LC + R>();
    else wait_vm_and_lds<0>();
    wg_barrier();
    read_frags(0, ldsA, ldsW, 0);

    auto run_tile = [&](auto full_tag) {
        auto one = [&](auto s_tag) {
            constexpr int S = decltype(s_tag)::value;
            if constexpr (S < NK) {
                if constexpr (decltype(full_tag)::value) slice(s_tag, std::true_type{});
                else if (jpos + NSW - 1 < J) slice(s_tag, std::true_type{});
                else slice(s_tag, std::false_type{});
            }
        };
        one(std::integral_constant<int, 0>{});
        one(std::integral_constant<int, 1>{});
        one(std::integral_constant<int, 2>{});
        one(std::integral_constant<int, 3>{});
    };
    static_assert(NK >= 1 && NK <= 4, "one to four K slices");
    for (int ti = 0; ti < t_count; ++ti) {
        // (the epilogue is instantiated behind either form of the tile so that the compiler, which places the waits
        // for the epilogue operands, can count the weight copies issued since they were requested)
        if (jpos + NK - 1 + NSW - 1 < J) {
            run_tile(std::true_type{});
            epilogue(ti);
        } else {
            run_tile(std::false_type{});
            epilogue(ti);
        }
        if (ti + 1 < t_count) request_epilogue_operands(ti + 1);
    }
}

template <int NK, bool HAS_OMASK>
static hipError_t launch_panel(const IgemmParams& p, hipStream_t stream) {
    const size_t smem = (size_t)(NK + 4) * 128 * 128 + 2 * kPanelMaxTiles * 128 * sizeof(float);
    auto kern = igemm_panel_kernel<NK, HAS_OMASK>;
    static std::atomic<size_t> granted{0};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, granted); e != hipSuccess) return e;
    SOL_LAUNCH(kern, dim3(p.total_tiles + p.red_blocks), dim3(256), smem, stream, p);
    return hipGetLastError();
}

// Whether the panel kernel can run this launch (tile-independent part; the caller has set ncls and the class).
bool igemm_panel_eligible(const IgemmParams& p) {
    if (p.ncls != 1 || p.addend_mask != nullptr || p.src_mask != nullptr) return false;
    const RowClass& rc = p.cls[0];
    if (rc.Th != 1 || rc.Tw != 1 || rc.h_mul != 1 || rc.w_mul != 1 || rc.h_off != 0 || rc.w_off != 0 || rc.Rh != p.Hs || rc.Rw != p.Ws) return false;
    if (rc.oh_mul != 1 || rc.ow_mul != 1 || rc.oh_off != 0 || rc.ow_off != 0 || rc.Rh != p.Hout || rc.Rw != p.Wout) return false;
    if (p.Cs != 64 && p.Cs != 128 && p.Cs != 192 && p.Cs != 256) return false;
    if (p.Nc % 128 != 0 || p.Nc < 256) return false;
    return (long long)rc.rows * p.Nc * 2 <= 0xffffffffLL;
}

// Chooses how many channel tiles a workgroup walks over (the launch has panels x groups workgroups, at most one
// wave of 256 where the shape allows; tiles_per_workgroup > 0 overrides, for tests and tuning).
// p.total_tiles (returned), p.panel_groups, p.panel_tiles are set here.
int plan_igemm_panel(IgemmParams& p, int tiles_per_workgroup) {
    const int panels = (p.cls[0].rows + 127) / 128, tiles_c = p.Nc / 128;
    p.total_tiles = 0;
    if (panels <= 0) return 0;
    int groups = 256 / panels;
    if (groups < 1) groups = 1;
    if (groups > tiles_c) groups = tiles_c;
    int per = tiles_per_workgroup > 0 ? tiles_per_workgroup : (tiles_c + groups - 1) / groups;
    if (per > tiles_c) per = tiles_c;
    if (per > kPanelMaxTiles) per = kPanelMaxTiles;
    groups = (tiles_c + per - 1) / per;
    p.tiles_c = tiles_c;
    p.panel_groups = groups;
    p.panel_tiles = per;
    p.total_tiles = panels * groups;
    p.cls[0].tile_begin = 0;
    return p.total_tiles;
}

// A launch planned by plan_igemm_panel (p.red_blocks workgroups more when it carries a split reduction along).
hipError_t launch_igemm_panel(const IgemmParams& p, hipStream_t stream) {
    if (p.total_tiles <= 0) return hipSuccess;
    const bool om = p.out_mask != nullptr;
    switch (p.Cs / 64) {
        case 1: return om ? launch_panel<1, true>(p, stream) : launch_panel<1, false>(p, stream);
        case 2: return om ? launch_panel<2, true>(p, stream) : launch_panel<2, false>(p, stream);
        case 3: return om ? launch_panel<3, true>(p, stream) : launch_panel<3, false>(p, stream);
        default: return om ? launch_panel<4, true>(p, stream) : launch_panel<4, false>(p, stream);
    }
}

}  // namespace sol
