// Weight gradient of the fused block as a split reduction over the N*Ho*Wo output pixels.
//
//   G[co][k] = sum_m g[m][co] * A[m][k],   g = ReLU ? (y > 0 ? dy : 0) : dy,
//   A = im2col(x) gathered on the fly, k = (kh, kw, ci) with ci fastest  (the KRSC order of dW)
//
// The reduction index m is the *strided* one of both operands in NHWC memory while an MFMA
// lane needs 8 consecutive reduction elements, so every thread loads an 8(m) x 8(channel)
// block of each operand with eight 16-byte loads, transposes it in registers and writes
// eight 16-byte pieces (one channel, 8 consecutive m) into LDS.  Each workgroup owns one
// 128(k) x 128(co) tile of G for one contiguous range of m ("split"); the fp32 tile goes to
// the workspace and `wgrad_reduce_kernel` adds the splits in a fixed order, scales by
// scale[co] and derives the affine-parameter gradients:
//   dshift[co] = sum_m g[m][co]            (column sums taken from the g blocks in registers)
//   dscale[co] = sum_k W[co][k] * G[co][k] (equals sum_m g * conv(x,W), no z needed)
#include "launch.h"
#include "reduce_rows.h"

namespace sol {

// rows r[0..7] hold 8 consecutive channels of 8 consecutive m; on return o[j] holds the 8
// consecutive m of channel j (16-bit elements).
__device__ __forceinline__ void transpose8x8_b16(const uintx4 (&r)[8], uintx4 (&o)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const unsigned a = r[2 * pr][j >> 1], b = r[2 * pr + 1][j >> 1];
            o[j][pr] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
        }
    }
}

// LDS tile: [128 rows (a channel or a k index)][16 chunks of 8 consecutive m].  The chunk
// index is XOR-ed with a row function chosen so that both the transposed 16-byte writes
// (fixed row % 8, varying row / 8) and the MFMA operand reads (32 consecutive rows) spread
// over all banks.
__device__ __forceinline__ int wg_swizzle(int row) { return ((row >> 3) ^ ((row & 7) << 1)) & 15; }

constexpr int WG_TILE = 128;     // tile edge along k, along co and along the reduction m
constexpr int WG_STAGE = 2 * WG_TILE * 16;   // 16-byte chunks per stage (two operand tiles)

template <bool VEC, bool MASK>
__global__ __launch_bounds__(256) void wgrad_bf16_kernel(const WgradParams p) {
    HIP_DYNAMIC_SHARED(uintx4, lds)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tiles = p.tiles_k * p.tiles_c;
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tk = t % p.tiles_k, tcn = t / p.tiles_k;
    const int k0 = tk * WG_TILE, co0 = tcn * WG_TILE;
    const int m_begin = split * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);
    const int iters = (m_end - m_begin + WG_TILE - 1) / WG_TILE;
    const bool do_shift = (tk == 0);

    // this thread's 8x8 blocks: chunk column cq (8 channels / 8 k) and m octet mq
    const int cq = tid & 15, mq = tid >> 4;
    const int kg = k0 + cq * 8;                 // first k of the x block
    int kh = 0, kw = 0, ci = 0;
    const bool k_ok = kg < p.K;
    if (VEC && k_ok) {
        const int tap = kg / p.C_in;
        ci = kg - tap * p.C_in;
        kh = tap / p.KW;
        kw = tap - kh * p.KW;
    }
    const int cg = co0 + cq * 8;                // first channel of the g block
    const bool c_ok = cg < p.C_out;
    const int HoWo = p.Ho * p.Wo;

    uintx4 xr[8], gr[8], yr[MASK ? 8 : 1];
    float colsum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) colsum[j] = 0.f;

    auto load_blocks = [&](int it) {
        const int mb = m_begin + it * WG_TILE + mq * 8;
        int n = mb / HoWo, rem = mb - n * HoWo;
        int ho = rem / p.Wo, wo = rem - ho * p.Wo;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int m = mb + e;
            const bool m_ok = m < m_end;
            if constexpr (VEC) {
                const int hi = ho * p.stride - p.pad + kh, wi = wo * p.stride - p.pad + kw;
                const bool ok = m_ok && k_ok && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
                const long long off = (((long long)n * p.H + hi) * p.W + wi) * p.C_in + ci;
                xr[e] = ok ? *reinterpret_cast<const uintx4*>(p.x + off) : uintx4{0, 0, 0, 0};
                const bool gok = m_ok && c_ok;
                const long long goff = (long long)m * p.C_out + cg;
                gr[e] = gok ? *reinterpret_cast<const uintx4*>(p.dy + goff) : uintx4{0, 0, 0, 0};
                if constexpr (MASK) yr[e] = gok ? *reinterpret_cast<const uintx4*>(p.y + goff) : uintx4{0, 0, 0, 0};
            } else {
                unsigned short xe[8], ge[8], ye[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xe[j] = 0;
                    ge[j] = 0;
                    ye[j] = 0;
                    const int k = kg + j;
                    if (m_ok && k < p.K) {
                        const int tap = k / p.C_in, c = k - tap * p.C_in;
                        const int t_h = tap / p.KW, t_w = tap - t_h * p.KW;
                        const int hi = ho * p.stride - p.pad + t_h, wi = wo * p.stride - p.pad + t_w;
                        if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
                            xe[j] = p.x[(((long long)n * p.H + hi) * p.W + wi) * p.C_in + c];
                    }
                    if (m_ok && cg + j < p.C_out) {
                        ge[j] = p.dy[(long long)m * p.C_out + cg + j];
                        if constexpr (MASK) ye[j] = p.y[(long long)m * p.C_out + cg + j];
                    }
                }
                xr[e] = uintx4{(unsigned)xe[0] | ((unsigned)xe[1] << 16), (unsigned)xe[2] | ((unsigned)xe[3] << 16),
                               (unsigned)xe[4] | ((unsigned)xe[5] << 16), (unsigned)xe[6] | ((unsigned)xe[7] << 16)};
                gr[e] = uintx4{(unsigned)ge[0] | ((unsigned)ge[1] << 16), (unsigned)ge[2] | ((unsigned)ge[3] << 16),
                               (unsigned)ge[4] | ((unsigned)ge[5] << 16), (unsigned)ge[6] | ((unsigned)ge[7] << 16)};
                if constexpr (MASK)
                    yr[e] = uintx4{(unsigned)ye[0] | ((unsigned)ye[1] << 16), (unsigned)ye[2] | ((unsigned)ye[3] << 16),
                                   (unsigned)ye[4] | ((unsigned)ye[5] << 16), (unsigned)ye[6] | ((unsigned)ye[7] << 16)};
            }
            if (++wo == p.Wo) {
                wo = 0;
                if (++ho == p.Ho) {
                    ho = 0;
                    ++n;
                }
            }
        }
    };

    auto store_blocks = [&](int stage) {
        uintx4* lx = lds + stage * WG_STAGE;     // x^T tile  [k row][m chunk]
        uintx4* lg = lx + WG_TILE * 16;          // g^T tile  [co row][m chunk]
        if constexpr (MASK) {
#pragma unroll
            for (int e = 0; e < 8; ++e) gr[e] = mask_where_positive(gr[e], yr[e]);
        }
        if (do_shift) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    colsum[2 * w] += __uint_as_float(gr[e][w] << 16);
                    colsum[2 * w + 1] += __uint_as_float(gr[e][w] & 0xffff0000u);
                }
        }
        uintx4 o[8];
        transpose8x8_b16(xr, o);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = cq * 8 + j;
            lx[row * 16 + (mq ^ wg_swizzle(row))] = o[j];
        }
        transpose8x8_b16(gr, o);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = cq * 8 + j;
            lg[row * 16 + (mq ^ wg_swizzle(row))] = o[j];
        }
    };

    // wave grid 2 (k) x 2 (co); every wave owns a 64 x 64 piece = 2 x 2 MFMA tiles
    const int wk = wave & 1, wcn = wave >> 1;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (iters > 0) {
        load_blocks(0);
        store_blocks(0);
    }
    __syncthreads();
    for (int it = 0; it < iters; ++it) {
        const bool more = it + 1 < iters;
        if (more) load_blocks(it + 1);
        const uintx4* lx = lds + (it & 1) * WG_STAGE;
        const uintx4* lg = lx + WG_TILE * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const int chunk = 2 * ks + (lane >> 5);
            bf16x8 xf[2], gf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wk * 64 + i * 32 + (lane & 31);
                xf[i] = __builtin_bit_cast(bf16x8, lx[row * 16 + (chunk ^ wg_swizzle(row))]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = wcn * 64 + j * 32 + (lane & 31);
                gf[j] = __builtin_bit_cast(bf16x8, lg[row * 16 + (chunk ^ wg_swizzle(row))]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[i], gf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_blocks((it + 1) & 1);
        __syncthreads();
    }

    // ---- partial tile: lane holds channel co (lane & 31) and, per quad q, 4 consecutive k ----
    float* part = p.partial + (long long)split * p.C_out * p.K;
    const bool vec_k = (p.K & 3) == 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int co = co0 + wcn * 64 + j * 32 + (lane & 31);
        if (co >= p.C_out) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int k = k0 + wk * 64 + i * 32 + 8 * q + 4 * (lane >> 5);
                if (k >= p.K) continue;
                float* dst = part + (long long)co * p.K + k;
                if (vec_k) {
                    *reinterpret_cast<floatx4*>(dst) =
                        floatx4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (k + e < p.K) dst[e] = acc[i][j][4 * q + e];
                }
            }
    }

    // ---- column sums of g for this split: add the 16 m-octet owners of every channel ------
    if (do_shift) {
        float* red = reinterpret_cast<float*>(lds);      // [16 mq][128 channels]; tiles are dead
#pragma unroll
        for (int j = 0; j < 8; ++j) red[mq * WG_TILE + cq * 8 + j] = colsum[j];
        __syncthreads();
        if (tid < WG_TILE && co0 + tid < p.C_out) {
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) s += red[q * WG_TILE + tid];
            p.dshift_partial[(long long)split * p.C_out + co0 + tid] = s;
        }
    }
}

// One workgroup per output channel: fixed-order sum over the splits, dW = scale * G,
// dscale = <W[co,:], G[co,:]> via wavefront shuffles, dshift = sum of the split column sums.
// VEC: the row reduction of reduce_rows.h with the whole workgroup on one row (K % 4 == 0, partial sums below 2 GB);
// else element by element.
template <bool VEC>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const ReduceParams p) {
    __shared__ float sums[kReduceLdsFloats];
    if constexpr (VEC) {
        reduce_rows_vec<256, 1>(p, blockIdx.x, gridDim.x, sums);
    } else {
        const int co = blockIdx.x, tid = threadIdx.x;
        const float sc = p.scale[co];
        const long long row = (long long)co * p.K;
        const long long split_stride = (long long)p.C_out * p.K;
        float dot = 0.f;
        for (int k = tid; k < p.K; k += 256) {
            float g = 0.f;
            for (int s = 0; s < p.splits; ++s) g += p.partial[s * split_stride + row + k];
            const float w = p.w_is_bf16 ? bf16_to_f32(reinterpret_cast<const bf16_t*>(p.W)[row + k])
                                        : reinterpret_cast<const float*>(p.W)[row + k];
            dot = fmaf(w, g, dot);
            const float d = sc * g;
            p.dW[row + k] = p.accumulate ? p.dW[row + k] + d : d;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        float mine = 0.f;
        for (int s2 = tid; s2 < p.splits; s2 += 256) mine += p.dshift_partial[(long long)s2 * p.C_out + co];
        float* ssum = sums;
        float* wsum = sums + 256;
        if ((tid & 63) == 0) wsum[tid >> 6] = dot;
        ssum[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            const float ds = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
            float db = 0.f;
            const int n = p.splits < 256 ? p.splits : 256;
            for (int s2 = 0; s2 < n; ++s2) db += ssum[s2];
            p.dscale[co] = p.accumulate ? p.dscale[co] + ds : ds;
            p.dshift[co] = p.accumulate ? p.dshift[co] + db : db;
        }
    }
}

hipError_t launch_wgrad(const WgradParams& p, bool vec, bool mask, hipStream_t stream) {
    const size_t smem = (size_t)2 * WG_STAGE * 16;
    const dim3 grid(p.tiles_k * p.tiles_c * p.splits), block(256);
    auto go = [&](auto kern) -> hipError_t {
        static std::atomic<size_t> granted{0};     // one per kernel instantiation (the lambda is generic)
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, granted); e != hipSuccess)
            return e;
        SOL_LAUNCH(kern, grid, block, smem, stream, p);
        return hipGetLastError();
    };
    if (vec) return mask ? go(wgrad_bf16_kernel<true, true>) : go(wgrad_bf16_kernel<true, false>);
    return mask ? go(wgrad_bf16_kernel<false, true>) : go(wgrad_bf16_kernel<false, false>);
}

hipError_t launch_wgrad_reduce(const ReduceParams& p, hipStream_t stream) {
    if (reduce_rows_ok(p)) SOL_LAUNCH(wgrad_reduce_kernel<true>, dim3(p.C_out), dim3(256), 0, stream, p);
    else SOL_LAUNCH(wgrad_reduce_kernel<false>, dim3(p.C_out), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace sol
