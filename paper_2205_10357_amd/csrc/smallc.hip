// Convolutions with very few input channels (the network stem: 7x7, stride 2, 3 -> 64 channels).
//
// With C_in = 3 a filter tap is 6 bytes of an NHWC row, so the implicit-GEMM kernels' 16-byte operand copies
// do not apply and their element-wise fallback is two orders of magnitude off the memory roofline of this
// layer (its output, not its arithmetic, is what must move).  Here:
//
//  * a preparation launch pads the image to 4 channels (8 bytes per pixel) and re-packs the weights into the
//    exact register image of the MFMA weight operand;
//  * K is ordered (kh, kw', ci) with kw' = 0..7 and ci = 0..3: one filter row is a "run" of 8 consecutive
//    padded pixels = 32 K elements = two 16-deep MFMA steps, K = 32 * KH (taps kw' >= KW and channel 3 carry
//    zero weights);
//  * a workgroup computes 128 consecutive output pixels of one output row for all 64 output channels.  It
//    stages the KH raw image rows it needs (128 * stride + 8 pixels each) in LDS; the MFMA pixel operand of
//    lane (pixel p, half h) at step (kh, half-run r) is the 16 bytes at pixel p*stride + 4r + 2h of row kh --
//    a plain aligned ds_read_b128 for stride 2, consecutive lanes 16 bytes apart: no im2col copy exists anywhere;
//  * all weight fragments of a wave (its 32 channels: 2*KH x 16 bytes per lane) stay in registers across the
//    tiles a workgroup processes;
//  * the accumulators hold 4 consecutive output channels per register group, so the epilogue (affine, ReLU,
//    one rounding) stores 8-byte pieces of NHWC rows directly.
#include <stdlib.h>

#include "launch.h"

namespace sol {

constexpr int SC_CO = 64;          // output channels (two 32-row MFMA tiles)
constexpr int SC_TILE = 128;       // output pixels of one row per workgroup tile
constexpr int SC_MAXKH = 8;
constexpr int SC_PK = 264;         // floats per channel row of a weight-gradient partial (256 columns + dshift + padding)

static inline __host__ __device__ int smallc_pad_blocks(long long pixels) { return (int)((pixels + 1023) / 1024); }

// ---- preparation: image -> 4 channels, weights -> operand image --------------------------------------
// Workgroups [0, pad_blocks) pad pixels (four per thread), the rest pack weights: element
// (step ks, channel co, half h, e) = W[co][kh = ks/2][kw' = 4*(ks&1) + 2*h + e/4][ci = e%4] or 0.
__global__ __launch_bounds__(256) void smallc_prepare_kernel(const SmallCParams p) {
    const long long pixels = (long long)p.N * p.H * p.W;
    const int pad_blocks = smallc_pad_blocks(pixels);
    if ((int)blockIdx.x < pad_blocks) {
        // four pixels per thread; with 3 channels they are 24 contiguous bytes (8-byte aligned) -> 32 bytes out
        const long long i4 = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
        if (i4 >= pixels) return;
        if (p.C_in == 3 && i4 + 4 <= pixels) {
            const uintx2* src = reinterpret_cast<const uintx2*>(p.x + i4 * 3);
            const uintx2 a = src[0], b = src[1], c = src[2];      // c0 c1 | c2 d0 | d1 d2 | e0 e1 | e2 f0 | f1 f2
            uintx4* dst = reinterpret_cast<uintx4*>(p.xp + i4 * 4);
            dst[0] = uintx4{a[0], a[1] & 0xffffu, (a[1] >> 16) | (b[0] << 16), b[0] >> 16};
            dst[1] = uintx4{b[1], c[0] & 0xffffu, (c[0] >> 16) | (c[1] << 16), c[1] >> 16};
            return;
        }
        for (long long i = i4; i < i4 + 4 && i < pixels; ++i) {
            const bf16_t* src = p.x + i * p.C_in;
            uintx2 v = {0u, 0u};
            v[0] = (uint32_t)src[0] | (p.C_in > 1 ? (uint32_t)src[1] << 16 : 0u);
            if (p.C_in > 2) v[1] = (uint32_t)src[2] | (p.C_in > 3 ? (uint32_t)src[3] << 16 : 0u);
            *reinterpret_cast<uintx2*>(p.xp + i * 4) = v;
        }
    } else {
        const int i = ((int)blockIdx.x - pad_blocks) * 256 + threadIdx.x;     // one 16-byte fragment piece per thread
        const int total = 2 * p.KH * SC_CO * 2;
        if (i >= total) return;
        const int h = i & 1, co = (i >> 1) % SC_CO, ks = (i >> 1) / SC_CO;
        const int kh = ks >> 1;
        unsigned short e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kw = 4 * (ks & 1) + 2 * h + (j >> 2), ci = j & 3;
            e[j] = (kw < p.KW && ci < p.C_in) ? p.Wt[(((long long)co * p.KH + kh) * p.KW + kw) * p.C_in + ci] : (unsigned short)0;
        }
        uintx4 v = {(uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                    (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16)};
        reinterpret_cast<uintx4*>(p.wp)[i] = v;
    }
}

// ---- forward ---------------------------------------------------------------------------------------------
template <int KH>
__global__ __launch_bounds__(256, 2) void smallc_fwd_kernel(const SmallCParams p) {
    constexpr int KS = 2 * KH;                       // 16-deep MFMA steps
    constexpr int PW = SC_TILE * 2 + 8;              // staged pixels per image row (stride 2)
    constexpr int OP = 17;                           // 8-byte pieces per staged output pixel (16 + 1 of padding)
    __shared__ __align__(16) uintx2 patch[KH * PW];  // [kh][pixel] 8 bytes each
    __shared__ __align__(16) uintx2 outs[SC_TILE * OP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int segs = (p.Wo + SC_TILE - 1) / SC_TILE;
    const int tiles = p.N * p.Ho * segs;

    // wave grid 2 (pixel halves of 64) x 2 (channel halves of 32): every wave keeps the weight fragments of its
    // 32 channels for all steps in registers -- lane (row co = 32*wc + lane%32, half lane/32), 16 bytes per step
    const int wp = wave & 1, wc = wave >> 1;
    uintx4 wf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        wf[ks] = reinterpret_cast<const uintx4*>(p.wp)[(ks * SC_CO + 32 * wc + (lane & 31)) * 2 + (lane >> 5)];
    // affine parameters of this lane's accumulator rows: co = 32*wc + 8*g + 4*(lane/32) + e
    floatx4 sc[4], sh[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int co = 32 * wc + 8 * g + 4 * (lane >> 5);
        sc[g] = *reinterpret_cast<const floatx4*>(p.scale + co);
        sh[g] = *reinterpret_cast<const floatx4*>(p.shift + co);
    }

    // the staged rows of a tile, fetched by this thread: flat element e = tid + 256*j of [KH][PW]
    constexpr int NL = (KH * PW + 255) / 256;
    auto fetch = [&](int t, uintx2 (&v)[NL]) {
        const int seg = t % segs, row = t / segs;
        const int ho = row % p.Ho, n = row / p.Ho;
        const int wi0 = seg * SC_TILE * 2 - p.pad;   // image column of staged pixel 0
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int e = tid + 256 * j;
            const int kh = e / PW, q = e - kh * PW;
            const int hi = ho * 2 - p.pad + kh, wi = wi0 + q;
            v[j] = uintx2{0u, 0u};
            if (e < KH * PW && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
                v[j] = *reinterpret_cast<const uintx2*>(p.xp + (((long long)n * p.H + hi) * p.W + wi) * 4);
        }
    };
    auto stage = [&](const uintx2 (&v)[NL]) {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int e = tid + 256 * j;
            if (e < KH * PW) patch[e] = v[j];
        }
    };

    uintx2 nextv[NL];
    int t = blockIdx.x;
    if (t < tiles) fetch(t, nextv);
    for (; t < tiles; t += gridDim.x) {
        const int seg = t % segs, row = t / segs;
        const int ho = row % p.Ho, n = row / p.Ho;
        const int wo0 = seg * SC_TILE;
        __syncthreads();                             // the previous tile's fragments have been read
        stage(nextv);
        __syncthreads();
        if (t + (int)gridDim.x < tiles) fetch(t + gridDim.x, nextv);      // in flight during this tile's arithmetic

        floatx16 acc[2];                             // pixel tiles j = 0, 1 of this wave's half
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
        const int pl0 = wp * 64 + (lane & 31);       // output pixel of this lane inside the tile (tile j adds 32)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int q = pl0 * 2 + 4 * (ks & 1) + 2 * (lane >> 5);
            const uintx2* rowp = &patch[(ks >> 1) * PW + q];
            const bf16x8 pf0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(rowp));
            const bf16x8 pf1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(rowp + 64));
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[ks]), pf0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[ks]), pf1, acc[1], 0, 0, 0);
        }

        // epilogue: affine, ReLU and the one rounding in the accumulator layout (4 consecutive channels per
        // register group), then through LDS so that every store instruction writes whole 128-byte pixel rows
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = fmaf(sc[g][e], acc[j][4 * g + e], sh[g][e]);
                    if (p.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                outs[(pl0 + 32 * j) * OP + 8 * wc + 2 * g + (lane >> 5)] =
                    uintx2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
            }
        __syncthreads();
        {
            bf16_t* dst = p.y + (((long long)n * p.Ho + ho) * p.Wo + wo0) * SC_CO;
            const int valid = p.Wo - wo0 < SC_TILE ? p.Wo - wo0 : SC_TILE;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = tid + 256 * j;               // 16-byte piece e of the tile's [128][64] bf16 rows
                const int px = e >> 3, c = e & 7;
                if (px < valid) {
                    const uintx2 a = outs[px * OP + 2 * c], b = outs[px * OP + 2 * c + 1];
                    store16_through(dst + px * SC_CO + c * 8, uintx4{a[0], a[1], b[0], b[1]});
                }
            }
        }
    }
}

bool smallc_fwd_supported(int C_in, int C_out, int KH, int KW, int stride) {
    return C_in >= 1 && C_in <= 4 && C_out == SC_CO && KH >= 1 && KH <= SC_MAXKH && KW >= 1 && KW <= 8 && stride == 2;
}

size_t smallc_padded_image_bytes(int N, int H, int W) { return (size_t)N * H * W * 4 * 2; }
size_t smallc_packed_weight_bytes(int KH) { return (size_t)2 * KH * SC_CO * 2 * 16; }

hipError_t launch_smallc_prepare(const SmallCParams& p, hipStream_t stream) {
    const long long pixels = (long long)p.N * p.H * p.W;
    const int pad_blocks = smallc_pad_blocks(pixels);
    const int pack_blocks = p.wp ? (2 * p.KH * SC_CO * 2 + 255) / 256 : 0;     // no packed weights wanted: pad only
    SOL_LAUNCH(smallc_prepare_kernel, dim3(pad_blocks + pack_blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int KH>
static hipError_t launch_smallc_fwd_kh(const SmallCParams& p, hipStream_t stream) {
    const int segs = (p.Wo + SC_TILE - 1) / SC_TILE;
    const long long tiles = (long long)p.N * p.Ho * segs;
    const long long cap = 512;                                 // two workgroups per compute unit
    const int grid = (int)(tiles < cap ? tiles : cap);         // several tiles per workgroup amortise the weight fetch
    SOL_LAUNCH(smallc_fwd_kernel<KH>, dim3(grid), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_smallc_fwd(const SmallCParams& p, hipStream_t stream) {
    switch (p.KH) {
        case 1: return launch_smallc_fwd_kh<1>(p, stream);
        case 2: return launch_smallc_fwd_kh<2>(p, stream);
        case 3: return launch_smallc_fwd_kh<3>(p, stream);
        case 4: return launch_smallc_fwd_kh<4>(p, stream);
        case 5: return launch_smallc_fwd_kh<5>(p, stream);
        case 6: return launch_smallc_fwd_kh<6>(p, stream);
        case 7: return launch_smallc_fwd_kh<7>(p, stream);
        case 8: return launch_smallc_fwd_kh<8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

// ---- weight gradient ------------------------------------------------------------------------------------
// G[k'][co] = sum over pixels of P[px][k'] * g[px][co], with P the same (kh, kw', ci) view of the staged image
// rows as in the forward kernel: for filter row kh, P[px][0..31] are the 64 bytes at pixel 2*px of staged row kh
// (rows of this "matrix" are 16 bytes apart and overlap).  The reduction index is the pixel, which is the row
// index of both operands in memory, so both MFMA operands come from transposing LDS reads (ds_read_b64_tr_b16:
// per 16 lanes a 4 x 16 block, 4 reduction rows x 16 columns).  A workgroup keeps its accumulators over all the
// row segments it processes and writes one fp32 partial [64 co][264] (32*KH gradient columns, column 256 = the
// column sum of g, i.e. dshift) at the end; smallc_wgrad_reduce_kernel adds the workgroups in a fixed order.
// Wave w owns filter-row slots 2w and 2w+1 for both channel tiles (2 x 2 register blocking: 8 transposing reads per
// 4 MFMAs); a slot without a filter row multiplies all-ones instead, and slot 7 (never a filter row) yields dshift.
template <int KH>
__global__ __launch_bounds__(256) void smallc_wgrad_kernel(const SmallCWgradParams p) {
    constexpr int PW = SC_TILE * 2 + 8;
    constexpr int GP = 160;                          // bytes per staged gradient row (128 + 32: the 4 rows of a
                                                     // transposing read fall into different banks)
    static_assert(KH <= 7, "filter-row slot 7 must be free for the column sums");
    __shared__ __align__(16) uintx2 patch[KH * PW];
    __shared__ __align__(16) unsigned char gt[SC_TILE * GP];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = lane >> 4, j = lane & 15;
    const int segs = (p.Wo + SC_TILE - 1) / SC_TILE;
    const int tiles = p.N * p.Ho * segs;

    // wave w owns filter-row slots 2w and 2w+1 for both channel tiles: acc[slot][channel tile]
    floatx16 acc[2][2];
#pragma unroll
    for (int v = 0; v < 16; ++v)
#pragma unroll
        for (int u = 0; u < 2; ++u) acc[u][0][v] = acc[u][1][v] = 0.f;

    // lane part of the transposing-read addresses (reduction row 8*(grp>>1) + (j>>2), column piece 16*(grp&1) + 4*(j&3))
    const int mrow = 8 * (grp >> 1) + (j >> 2);
    const unsigned char* gbase = gt + mrow * GP + (16 * (grp & 1) + 4 * (j & 3)) * 2;
    const unsigned char* pbase = reinterpret_cast<const unsigned char*>(patch) + mrow * 16 + 32 * (grp & 1) + 8 * (j & 3);
    // A slot whose filter row does not exist multiplies an all-ones operand instead (its reads go to the last real
    // row and are discarded): the step loop then has no branch, and the ones-product is the column sum of g.
    const unsigned char* prow[2];
    bool use_ones[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int kh = 2 * wave + u;
        use_ones[u] = kh >= KH;
        prow[u] = pbase + (kh < KH ? kh : KH - 1) * PW * 8;
    }

    // the operands of a tile as fetched by this thread: 4 gradient pieces (16 bytes) and NL image pixels (8 bytes)
    constexpr int NL = (KH * PW + 255) / 256;
    auto fetch = [&](int t, uintx4 (&gv)[4], uintx2 (&xv)[NL]) {
        const int seg = t % segs, row = t / segs;
        const int ho = row % p.Ho, n = row / p.Ho;
        const int wo0 = seg * SC_TILE;
        const int wi0 = wo0 * 2 - p.pad;
        const int valid = p.Wo - wo0 < SC_TILE ? p.Wo - wo0 : SC_TILE;
        // gradient rows: 128 pixels x 64 channels; rows past the end of the image row are zero
        const bf16_t* gsrc = p.dy + (((long long)n * p.Ho + ho) * p.Wo + wo0) * SC_CO;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int e = tid + 256 * jj;
            const int px = e >> 3, c = e & 7;
            gv[jj] = uintx4{0u, 0u, 0u, 0u};
            if (px < valid) gv[jj] = *reinterpret_cast<const uintx4*>(gsrc + px * SC_CO + c * 8);
        }
        // image rows, as in the forward kernel
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            const int e = tid + 256 * jj;
            const int kh = e / PW, q = e - kh * PW;
            const int hi = ho * 2 - p.pad + kh, wi = wi0 + q;
            xv[jj] = uintx2{0u, 0u};
            if (e < KH * PW && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
                xv[jj] = *reinterpret_cast<const uintx2*>(p.xp + (((long long)n * p.H + hi) * p.W + wi) * 4);
        }
    };

    uintx4 gnext[4];
    uintx2 xnext[NL];
    int t = blockIdx.x;
    if (t < tiles) fetch(t, gnext, xnext);
    for (; t < tiles; t += gridDim.x) {
        __syncthreads();                             // the previous tile has been read
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int e = tid + 256 * jj;
            *reinterpret_cast<uintx4*>(gt + (e >> 3) * GP + (e & 7) * 16) = gnext[jj];
        }
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            const int e = tid + 256 * jj;
            if (e < KH * PW) patch[e] = xnext[jj];
        }
        __syncthreads();
        if (t + (int)gridDim.x < tiles) fetch(t + gridDim.x, gnext, xnext);   // in flight during this tile's arithmetic

#pragma unroll
        for (int s = 0; s < SC_TILE / 16; ++s) {     // no branch in here: see `use_ones`
            bf16x8 gf[2], pf[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const unsigned char* a = gbase + 16 * s * GP + 64 * c;
                const uintx2 g0 = lds_read_tr_b64(a), g1 = lds_read_tr_b64(a + 4 * GP);
                gf[c] = __builtin_bit_cast(bf16x8, uintx4{g0[0], g0[1], g1[0], g1[1]});
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const unsigned char* a = prow[u] + 16 * s * 16;
                const uintx2 p0 = lds_read_tr_b64(a), p1 = lds_read_tr_b64(a + 64);
                uintx4 pv = {p0[0], p0[1], p1[0], p1[1]};
#pragma unroll
                for (int e = 0; e < 4; ++e) pv[e] = use_ones[u] ? 0x3f803f80u : pv[e];
                pf[u] = __builtin_bit_cast(bf16x8, pv);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    acc[u][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[u], gf[c], acc[u][c], 0, 0, 0);
        }
    }

    // partial of this workgroup: [co][SC_PK], lane = channel (lane & 31), 4 consecutive k' per register group
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        float* part = p.partial + (long long)blockIdx.x * SC_CO * SC_PK + (long long)(32 * c + (lane & 31)) * SC_PK;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int kh = 2 * wave + u;
            if (kh < KH) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<floatx4*>(part + kh * 32 + 8 * g + 4 * (lane >> 5)) =
                        floatx4{acc[u][c][4 * g], acc[u][c][4 * g + 1], acc[u][c][4 * g + 2], acc[u][c][4 * g + 3]};
            }
        }
        // slot 7 (wave 3, u = 1) never has a filter row: every row of its ones-product is the column sum of g
        if (wave == 3 && lane < 32) part[256] = acc[1][c][0];
    }
}

// One workgroup of 1024 threads per output channel: thread (q, k') sums every fourth partial of column k' (more
// loads in flight than 256 threads give), the four sums are added in a fixed order; dW = scale * G on the real
// taps and channels, dscale = <W[co,:], G[co,:]>, dshift = sum of the column sums (column 256, thread 255).
__global__ __launch_bounds__(1024) void smallc_wgrad_reduce_kernel(const SmallCWgradParams p) {
    __shared__ float quarter[4][SC_PK];
    __shared__ float red[256];
    const int co = blockIdx.x, tid = threadIdx.x & 255, q = threadIdx.x >> 8;
    const long long stride = (long long)SC_CO * SC_PK;
    const bool col_ok = tid < 32 * p.KH || tid == 255;
    const int col = tid == 255 ? 256 : tid;
    if (col_ok) {
        const float* src = p.partial + (long long)co * SC_PK + col;
        float g = 0.f;
        int b = q;
        for (; b + 28 < p.nparts; b += 32) {           // 8 loads in flight, fixed add order
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = src[(b + 4 * u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) g += a[u];
        }
        for (; b < p.nparts; b += 4) g += src[b * stride];
        quarter[q][col] = g;
    }
    __syncthreads();
    float g = 0.f, dot = 0.f;
    if (q == 0 && col_ok) g = (quarter[0][col] + quarter[1][col]) + (quarter[2][col] + quarter[3][col]);
    const int kh = tid >> 5, kw = (tid & 31) >> 2, ci = tid & 3;
    if (q == 0 && tid < 32 * p.KH && kw < p.KW && ci < p.C_in) {
        const long long o = (((long long)co * p.KH + kh) * p.KW + kw) * p.C_in + ci;
        dot = bf16_to_f32(p.Wt[o]) * g;
        const float d = p.scale[co] * g;
        p.dW[o] = p.accumulate ? p.dW[o] + d : d;
    }
    if (q == 0) red[tid] = dot;
    __syncthreads();
    if (q == 0 && tid < 64) {
        float v = (red[tid] + red[tid + 64]) + (red[tid + 128] + red[tid + 192]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if (tid == 0) p.dscale[co] = p.accumulate ? p.dscale[co] + v : v;
    }
    if (q == 0 && tid == 255) p.dshift[co] = p.accumulate ? p.dshift[co] + g : g;
}

bool smallc_wgrad_supported(int C_in, int C_out, int KH, int KW, int stride) {
    return smallc_fwd_supported(C_in, C_out, KH, KW, stride) && KH <= 7;
}

int smallc_wgrad_parts(int N, int Ho, int Wo) {
    const long long tiles = (long long)N * Ho * ((Wo + SC_TILE - 1) / SC_TILE);
    return (int)(tiles < 256 ? tiles : 256);         // one workgroup per compute unit keeps the partials small
}
size_t smallc_wgrad_partial_bytes(int nparts) { return (size_t)nparts * SC_CO * SC_PK * 4; }

template <int KH>
static hipError_t launch_smallc_wgrad_kh(const SmallCWgradParams& p, hipStream_t stream) {
    SOL_LAUNCH(smallc_wgrad_kernel<KH>, dim3(p.nparts), dim3(256), 0, stream, p);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    SOL_LAUNCH(smallc_wgrad_reduce_kernel, dim3(SC_CO), dim3(1024), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_smallc_wgrad(const SmallCWgradParams& p, hipStream_t stream) {
    switch (p.KH) {
        case 1: return launch_smallc_wgrad_kh<1>(p, stream);
        case 2: return launch_smallc_wgrad_kh<2>(p, stream);
        case 3: return launch_smallc_wgrad_kh<3>(p, stream);
        case 4: return launch_smallc_wgrad_kh<4>(p, stream);
        case 5: return launch_smallc_wgrad_kh<5>(p, stream);
        case 6: return launch_smallc_wgrad_kh<6>(p, stream);
        case 7: return launch_smallc_wgrad_kh<7>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sol
