// Implicit-GEMM convolution on bf16 MFMA (v_mfma_f32_32x32x16_bf16, fp32 accumulate) for
// gfx950, used by the forward pass of the fused block and by its data gradient.
//
// GEMM view:  out[pixel][c] = sum_k  G[pixel][k] * Wm[c][k]
//   G      gathered on the fly from an NHWC activation (im2col never exists in memory);
//          k = (tap_h, tap_w, source channel), source channel fastest
//   Wm     weight matrix with K-contiguous rows (KRSC weights as they are for the forward
//          pass; a re-packed, scale-folded copy per row class for the data gradient)
// Both operands are staged through LDS in 64-deep K slices (16-byte chunks, XOR-swizzled so
// that the 16-byte reads of the MFMA operands spread over all banks), double buffered, with
// the next slice prefetched into registers while the current one is multiplied.
// The weight tile is the MFMA "A" operand and the pixel tile the "B" operand, so each lane
// ends up with 4 consecutive channels of one pixel per accumulator quad and the epilogue
// (affine, residual / addend, ReLU, one rounding to bf16) stores 8-byte pieces of NHWC rows.
#include "launch.h"

namespace sol {

__device__ __forceinline__ int lds_swizzle(int row) { return (row + (row >> 3)) & 7; }

template <int BP, int BC, int WP, int WC, bool VEC, bool MASK>
__global__ __launch_bounds__(256) void igemm_bf16_kernel(const IgemmParams p) {
    static_assert(WP * WC == 4, "four waves per workgroup");
    constexpr int AP = BP / 32;            // 16-byte chunks per thread, pixel tile
    constexpr int AC = BC / 32;            // 16-byte chunks per thread, weight tile
    constexpr int TP = BP / WP / 32;       // MFMA tiles per wave along pixels
    constexpr int TC = BC / WC / 32;       // MFMA tiles per wave along channels
    constexpr int STAGE = (BP + BC) * 8;   // chunks per pipeline stage

    HIP_DYNAMIC_SHARED(uintx4, lds)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tc = bid % p.tiles_c;
    int tp = bid / p.tiles_c;
    int cidx = 0;
#pragma unroll
    for (int i = 1; i < kMaxClasses; ++i)
        if (i < p.ncls && tp >= p.cls[i].tile_begin) cidx = i;
    const RowClass rc = p.cls[cidx];
    tp -= rc.tile_begin;
    const int row0 = tp * BP, ch0 = tc * BC;
    const int K = rc.Th * rc.Tw * p.Cs;
    const int nk = (K + 63) >> 6;
    const int img_rows = rc.Rh * rc.Rw;
    const bf16_t* wmat = p.wmat + rc.b_off;

    // ---- per-thread gather state: which rows / which 8-wide K chunk this thread stages ----
    const int c8 = tid & 7, r0 = tid >> 3;
    int h0[AP], w0[AP], img[AP];
#pragma unroll
    for (int i = 0; i < AP; ++i) {
        const int r = row0 + r0 + 32 * i;
        if (r < rc.rows) {
            const int n = (int)fast_div((uint32_t)r, rc.div_img), rem = r - n * img_rows;
            const int rh = (int)fast_div((uint32_t)rem, rc.div_rw), rw = rem - rh * rc.Rw;
            h0[i] = rh * rc.h_mul + rc.h_off;
            w0[i] = rw * rc.w_mul + rc.w_off;
            img[i] = n * p.Hs * p.Ws * p.Cs;
        } else {
            h0[i] = -(1 << 24);
            w0[i] = 0;
            img[i] = 0;
        }
    }
    // position of this thread's chunk inside K: tap (th, tw) and first channel cc
    int th, tw, cc;
    {
        const int k = c8 * 8;
        const int tap = k / p.Cs;
        cc = k - tap * p.Cs;
        th = tap / rc.Tw;
        tw = tap - th * rc.Tw;
    }

    uintx4 a_reg[AP], m_reg[MASK ? AP : 1], b_reg[AC];

    auto load_slice = [&](int kt) {
        if constexpr (VEC) {
            const bool kv = th < rc.Th;
            const int dh = th * rc.tap_step, dw = tw * rc.tap_step;
#pragma unroll
            for (int i = 0; i < AP; ++i) {
                const int h = h0[i] + dh, w = w0[i] + dw;
                const bool ok = kv && (unsigned)h < (unsigned)p.Hs && (unsigned)w < (unsigned)p.Ws;
                const int off = img[i] + (h * p.Ws + w) * p.Cs + cc;
                a_reg[i] = ok ? *reinterpret_cast<const uintx4*>(p.src + off) : uintx4{0, 0, 0, 0};
                if constexpr (MASK)
                    m_reg[i] = ok ? *reinterpret_cast<const uintx4*>(p.src_mask + off) : uintx4{0, 0, 0, 0};
            }
            const int kb = kt * 64 + c8 * 8;
#pragma unroll
            for (int i = 0; i < AC; ++i) {
                const int ch = ch0 + r0 + 32 * i;
                const bool ok = kv && ch < p.Nc;
                b_reg[i] = ok ? *reinterpret_cast<const uintx4*>(wmat + (long long)ch * K + kb)
                              : uintx4{0, 0, 0, 0};
            }
        } else {
            // element-wise gather for channel counts that are not a multiple of 8
            const int kb = kt * 64 + c8 * 8;
#pragma unroll
            for (int i = 0; i < AP; ++i) {
                unsigned short e[8], m[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = kb + j;
                    e[j] = 0;
                    m[j] = 0;
                    if (k < K) {
                        const int tap = k / p.Cs, c = k - tap * p.Cs;
                        const int t_h = tap / rc.Tw, t_w = tap - t_h * rc.Tw;
                        const int h = h0[i] + t_h * rc.tap_step, w = w0[i] + t_w * rc.tap_step;
                        if ((unsigned)h < (unsigned)p.Hs && (unsigned)w < (unsigned)p.Ws) {
                            const int off = img[i] + (h * p.Ws + w) * p.Cs + c;
                            e[j] = p.src[off];
                            if constexpr (MASK) m[j] = p.src_mask[off];
                        }
                    }
                }
                a_reg[i] = uintx4{(unsigned)e[0] | ((unsigned)e[1] << 16), (unsigned)e[2] | ((unsigned)e[3] << 16),
                                  (unsigned)e[4] | ((unsigned)e[5] << 16), (unsigned)e[6] | ((unsigned)e[7] << 16)};
                if constexpr (MASK)
                    m_reg[i] = uintx4{(unsigned)m[0] | ((unsigned)m[1] << 16), (unsigned)m[2] | ((unsigned)m[3] << 16),
                                      (unsigned)m[4] | ((unsigned)m[5] << 16), (unsigned)m[6] | ((unsigned)m[7] << 16)};
            }
#pragma unroll
            for (int i = 0; i < AC; ++i) {
                const int ch = ch0 + r0 + 32 * i;
                unsigned short e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = kb + j;
                    e[j] = (ch < p.Nc && k < K) ? wmat[(long long)ch * K + k] : (unsigned short)0;
                }
                b_reg[i] = uintx4{(unsigned)e[0] | ((unsigned)e[1] << 16), (unsigned)e[2] | ((unsigned)e[3] << 16),
                                  (unsigned)e[4] | ((unsigned)e[5] << 16), (unsigned)e[6] | ((unsigned)e[7] << 16)};
            }
        }
    };

    auto advance_chunk = [&]() {   // move this thread's chunk 64 elements further along K
        cc += 64;
        while (cc >= p.Cs) {
            cc -= p.Cs;
            if (++tw == rc.Tw) {
                tw = 0;
                ++th;
            }
        }
    };

    auto store_slice = [&](int stage) {
        uintx4* lp = lds + stage * STAGE;
        uintx4* lw = lp + BP * 8;
#pragma unroll
        for (int i = 0; i < AP; ++i) {
            const int r = r0 + 32 * i;
            uintx4 v = a_reg[i];
            if constexpr (MASK) v = mask_where_positive(v, m_reg[i]);
            lp[r * 8 + (c8 ^ lds_swizzle(r))] = v;
        }
#pragma unroll
        for (int i = 0; i < AC; ++i) {
            const int r = r0 + 32 * i;
            lw[r * 8 + (c8 ^ lds_swizzle(r))] = b_reg[i];
        }
    };

    const int wp = wave % WP, wc = wave / WP;
    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (nk > 0) {
        load_slice(0);
        if constexpr (VEC) advance_chunk();
        store_slice(0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) {
            load_slice(kt + 1);
            if constexpr (VEC) advance_chunk();
        }
        const uintx4* lp = lds + (kt & 1) * STAGE;
        const uintx4* lw = lp + BP * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int chunk = 2 * ks + (lane >> 5);
            bf16x8 wf[TC], pf[TP];
#pragma unroll
            for (int i = 0; i < TC; ++i) {
                const int r = wc * (BC / WC) + i * 32 + (lane & 31);
                wf[i] = __builtin_bit_cast(bf16x8, lw[r * 8 + (chunk ^ lds_swizzle(r))]);
            }
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const int r = wp * (BP / WP) + j * 32 + (lane & 31);
                pf[j] = __builtin_bit_cast(bf16x8, lp[r * 8 + (chunk ^ lds_swizzle(r))]);
            }
#pragma unroll
            for (int i = 0; i < TC; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], pf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_slice((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds pixel (lane & 31) of each pixel sub-tile and, per accumulator
    //      quad q, channels 8*q + 4*(lane >> 5) .. +3 of each channel sub-tile ----------------
    const bool vec_out = (p.Nc & 3) == 0;
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int r = row0 + wp * (BP / WP) + j * 32 + (lane & 31);
        if (r >= rc.rows) continue;
        const int n = (int)fast_div((uint32_t)r, rc.div_img), rem = r - n * img_rows;
        const int rh = (int)fast_div((uint32_t)rem, rc.div_rw), rw = rem - rh * rc.Rw;
        const long long opix = ((long long)n * p.Hout + (rh * rc.oh_mul + rc.oh_off)) * p.Wout +
                               (rw * rc.ow_mul + rc.ow_off);
        const long long obase = opix * p.Nc;
#pragma unroll
        for (int i = 0; i < TC; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = ch0 + wc * (BC / WC) + i * 32 + 8 * q + 4 * (lane >> 5);
                if (ch >= p.Nc) continue;
                float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                if (vec_out) {
                    if (p.scale) {
                        const floatx4 sc = *reinterpret_cast<const floatx4*>(p.scale + ch);
                        const floatx4 sh = *reinterpret_cast<const floatx4*>(p.shift + ch);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaf(sc[e], v[e], sh[e]);
                    }
                    if (p.addend) {
                        uintx2 a = *reinterpret_cast<const uintx2*>(p.addend + obase + ch);
                        if (p.addend_mask)
                            a = mask_where_positive(a, *reinterpret_cast<const uintx2*>(p.addend_mask + obase + ch));
                        v[0] += __uint_as_float(a[0] << 16);
                        v[1] += __uint_as_float(a[0] & 0xffff0000u);
                        v[2] += __uint_as_float(a[1] << 16);
                        v[3] += __uint_as_float(a[1] & 0xffff0000u);
                    }
                    if (p.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    uintx2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                    if (p.out_mask)
                        o = mask_where_positive(o, *reinterpret_cast<const uintx2*>(p.out_mask + obase + ch));
                    *reinterpret_cast<uintx2*>(p.out + obase + ch) = o;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (ch + e >= p.Nc) break;
                        float t = v[e];
                        if (p.scale) t = fmaf(p.scale[ch + e], t, p.shift[ch + e]);
                        if (p.addend) {
                            const bf16_t a = p.addend[obase + ch + e];
                            const bool keep = !p.addend_mask || (short)p.addend_mask[obase + ch + e] > 0;
                            if (keep) t += bf16_to_f32(a);
                        }
                        if (p.relu) t = t > 0.f ? t : 0.f;
                        if (p.out_mask && !((short)p.out_mask[obase + ch + e] > 0)) t = 0.f;
                        p.out[obase + ch + e] = f32_to_bf16(t);
                    }
                }
            }
        }
    }
}

// -------------------------------------------------------------------------------- launch
template <int BP, int BC, int WP, int WC>
static hipError_t launch_tile(const IgemmParams& p, bool vec, bool mask, hipStream_t stream) {
    const size_t smem = (size_t)2 * (BP + BC) * 8 * 16;
    const dim3 grid(p.total_tiles), block(256);
    auto go = [&](auto kern) -> hipError_t {
        static std::atomic<size_t> granted{0};     // one per kernel instantiation (the lambda is generic)
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, granted); e != hipSuccess)
            return e;
        SOL_LAUNCH(kern, grid, block, smem, stream, p);
        return hipGetLastError();
    };
    if (vec) return mask ? go(igemm_bf16_kernel<BP, BC, WP, WC, true, true>)
                         : go(igemm_bf16_kernel<BP, BC, WP, WC, true, false>);
    return mask ? go(igemm_bf16_kernel<BP, BC, WP, WC, false, true>)
                : go(igemm_bf16_kernel<BP, BC, WP, WC, false, false>);
}

// tile: 0 = 128 pixels x 128 channels, 1 = 256 x 128, 2 = 128 x 64, 3 = 64 x 64
hipError_t launch_igemm(const IgemmParams& p, int tile, bool vec, bool mask, hipStream_t stream) {
    if (p.total_tiles <= 0) return hipSuccess;
    switch (tile) {
        case 0: return launch_tile<128, 128, 2, 2>(p, vec, mask, stream);
        case 1: return launch_tile<256, 128, 2, 2>(p, vec, mask, stream);
        case 2: return launch_tile<128, 64, 2, 2>(p, vec, mask, stream);
        default: return launch_tile<64, 64, 2, 2>(p, vec, mask, stream);
    }
}

void igemm_tile_shape(int tile, int* bp, int* bc) {
    static const int shapes[4][2] = {{128, 128}, {256, 128}, {128, 64}, {64, 64}};
    const int t = (tile < 0 || tile > 3) ? 3 : tile;
    *bp = shapes[t][0];
    *bc = shapes[t][1];
}

}  // namespace sol
