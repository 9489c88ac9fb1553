// Small memory-bound helpers around the two GEMM kernels: weight re-packing for the data
// gradient, the masked gradient copy (dres), the L1-loss gradient and the stem max-pool.
#include "launch.h"
#include "classes.h"
#include "pack_tile.h"

namespace sol {

// out[class][ci][(jh*Tw + jw)*C_out + co] = bf16(scale[co] * W[co][kh][kw][ci]); one thread per
// weight element, indexed so that writes are contiguous in co.
__global__ __launch_bounds__(256) void pack_dgrad_weights_kernel(const PackParams p) {
    const long long total = (long long)p.C_out * p.KH * p.KW * p.C_in;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int co = (int)(idx % p.C_out);
    long long r = idx / p.C_out;
    const int ci = (int)(r % p.C_in);
    r /= p.C_in;
    const int kw = (int)(r % p.KW);
    const int kh = (int)(r / p.KW);
    const int s = p.stride;
    const int ph = ((kh - p.pad) % s + s) % s, pw = ((kw - p.pad) % s + s) % s;
    int fh, fw;
    const int Th = class_taps(p.KH, s, p.pad, ph, &fh), Tw = class_taps(p.KW, s, p.pad, pw, &fw);
    const long long off = class_weight_offset(p.C_in, p.C_out, p.KH, p.KW, s, p.pad, ph, pw);
    const int jh = (kh - fh) / s, jw = (kw - fw) / s;
    const float w = bf16_to_f32(p.W[(((long long)co * p.KH + kh) * p.KW + kw) * p.C_in + ci]);
    p.out[off + ((long long)ci * Th * Tw + (jh * Tw + jw)) * p.C_out + co] = f32_to_bf16(p.scale[co] * w);
}

// Same re-packing for channel counts that are multiples of 64: one workgroup per (tap, 64 co, 64 ci) tile.
__global__ __launch_bounds__(256) void pack_dgrad_weights_tiled_kernel(const PackParams p) {
    __shared__ __align__(16) bf16_t tile[64 * kPackTilePitch];
    pack_dgrad_weights_tile(p, (int)blockIdx.x, tile);
}

template <typename T>
__global__ __launch_bounds__(256) void masked_copy_kernel(const T* dy, const T* y, T* dres, long long numel) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= numel) return;
    if constexpr (sizeof(T) == 2) {
        dres[i] = (!y || (short)y[i] > 0) ? dy[i] : (T)0;
    } else {
        dres[i] = (!y || y[i] > 0.f) ? dy[i] : (T)0;
    }
}

// bf16, 8 elements (16 bytes) per thread; the last thread finishes a ragged tail element by element
__global__ __launch_bounds__(256) void masked_copy_bf16x8_kernel(const bf16_t* dy, const bf16_t* y, bf16_t* dres,
                                                                 long long numel) {
    const long long i8 = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i8 >= numel) return;
    if (i8 + 8 <= numel) {
        const uintx4 g = *reinterpret_cast<const uintx4*>(dy + i8);
        store16_through(dres + i8, y ? mask_where_positive(g, *reinterpret_cast<const uintx4*>(y + i8)) : g);
    } else {
        for (long long i = i8; i < numel; ++i) dres[i] = (!y || (short)y[i] > 0) ? dy[i] : (bf16_t)0;
    }
}

// dy = sign(y - t) / numel, optionally zero where y <= 0.  bf16: 8 elements (16 bytes) per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void l1_grad_kernel(const void* yv, const void* tv, void* dyv, long long numel,
                                                      float inv, int mask_by_y) {
    auto grad = [&](float y, float t) {
        float d = y > t ? inv : (y < t ? -inv : 0.f);
        if (mask_by_y && !(y > 0.f)) d = 0.f;
        return d;
    };
    if constexpr (BF16) {
        const long long i8 = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
        if (i8 >= numel) return;
        const bf16_t* yb = reinterpret_cast<const bf16_t*>(yv);
        const bf16_t* tb = reinterpret_cast<const bf16_t*>(tv);
        bf16_t* db = reinterpret_cast<bf16_t*>(dyv);
        if (i8 + 8 <= numel) {
            const uintx4 y4 = *reinterpret_cast<const uintx4*>(yb + i8);
            const uintx4 t4 = *reinterpret_cast<const uintx4*>(tb + i8);
            uintx4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = grad(__uint_as_float(y4[e] << 16), __uint_as_float(t4[e] << 16));
                const float hi = grad(__uint_as_float(y4[e] & 0xffff0000u), __uint_as_float(t4[e] & 0xffff0000u));
                o[e] = pack_bf16x2(lo, hi);
            }
            store16_through(db + i8, o);
        } else {
            for (long long i = i8; i < numel; ++i) db[i] = f32_to_bf16(grad(bf16_to_f32(yb[i]), bf16_to_f32(tb[i])));
        }
    } else {
        const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
        if (i >= numel) return;
        reinterpret_cast<float*>(dyv)[i] = grad(reinterpret_cast<const float*>(yv)[i], reinterpret_cast<const float*>(tv)[i]);
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void maxpool_kernel(const void* xv, void* yv, int N, int H, int W, int C, int k,
                                                      int stride, int pad, int Ho, int Wo) {
    const long long total = (long long)N * Ho * Wo * C;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % C);
    long long pix = idx / C;
    const int wo = (int)(pix % Wo);
    pix /= Wo;
    const int ho = (int)(pix % Ho);
    const int n = (int)(pix / Ho);
    float m = -INFINITY;
    for (int kh = 0; kh < k; ++kh) {
        const int hi = ho * stride - pad + kh;
        if ((unsigned)hi >= (unsigned)H) continue;
        for (int kw = 0; kw < k; ++kw) {
            const int wi = wo * stride - pad + kw;
            if ((unsigned)wi >= (unsigned)W) continue;
            const long long o = (((long long)n * H + hi) * W + wi) * C + c;
            const float v = BF16 ? bf16_to_f32(reinterpret_cast<const bf16_t*>(xv)[o])
                                 : reinterpret_cast<const float*>(xv)[o];
            m = v > m ? v : m;
        }
    }
    if constexpr (BF16) reinterpret_cast<bf16_t*>(yv)[idx] = f32_to_bf16(m);
    else reinterpret_cast<float*>(yv)[idx] = m;
}

// Data gradient of a strided block, input pixels that no filter tap reaches (1x1 / stride 2: three of four): their
// gradient is the addend (optionally gated) or zero, then the optional output mask.  One thread per (pixel, 8
// channels); pixels that some tap reaches belong to the GEMM launch and are left alone.
__global__ __launch_bounds__(256) void untouched_pixels_kernel(bf16_t* dx, const bf16_t* addend, const bf16_t* addend_mask,
                                                               const bf16_t* out_mask, int N, int H, int W, int C, int KH,
                                                               int KW, int stride, int pad) {
    const int c8 = C >> 3;
    const long long total = (long long)N * H * W * c8;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long pix = idx / c8;
    const int wi = (int)(pix % W), hi = (int)((pix / W) % H);
    int f;
    if (class_taps(KH, stride, pad, hi % stride, &f) > 0 && class_taps(KW, stride, pad, wi % stride, &f) > 0) return;
    uintx4 v = {0u, 0u, 0u, 0u};
    if (addend) {
        v = *reinterpret_cast<const uintx4*>(addend + idx * 8);
        if (addend_mask) v = mask_where_positive(v, *reinterpret_cast<const uintx4*>(addend_mask + idx * 8));
    }
    if (out_mask) v = mask_where_positive(v, *reinterpret_cast<const uintx4*>(out_mask + idx * 8));
    store16_through(dx + idx * 8, v);
}

static inline unsigned blocks_for(long long total) { return (unsigned)((total + 255) / 256); }

hipError_t launch_untouched_pixels(void* dx, const void* addend, const void* addend_mask, const void* out_mask, int N,
                                   int H, int W, int C, int KH, int KW, int stride, int pad, hipStream_t s) {
    const long long total = (long long)N * H * W * (C >> 3);
    if (total <= 0) return hipSuccess;
    SOL_LAUNCH(untouched_pixels_kernel, dim3(blocks_for(total)), dim3(256), 0, s, (bf16_t*)dx,
                       (const bf16_t*)addend, (const bf16_t*)addend_mask, (const bf16_t*)out_mask, N, H, W, C, KH, KW,
                       stride, pad);
    return hipGetLastError();
}

hipError_t launch_pack_dgrad_weights(const PackParams& p, hipStream_t s) {
    const long long total = (long long)p.C_out * p.KH * p.KW * p.C_in;
    if ((p.C_in & 63) == 0 && (p.C_out & 63) == 0)
        SOL_LAUNCH(pack_dgrad_weights_tiled_kernel, dim3((unsigned)pack_tile_count(p)), dim3(256), 0, s, p);
    else
        SOL_LAUNCH(pack_dgrad_weights_kernel, dim3(blocks_for(total)), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_masked_copy(int dtype, const void* dy, const void* y, void* dres, long long numel, hipStream_t s) {
    if (numel <= 0) return hipSuccess;
    if (dtype == 1)
        SOL_LAUNCH(masked_copy_bf16x8_kernel, dim3(blocks_for((numel + 7) / 8)), dim3(256), 0, s,
                   (const bf16_t*)dy, (const bf16_t*)y, (bf16_t*)dres, numel);
    else
        SOL_LAUNCH(masked_copy_kernel<float>, dim3(blocks_for(numel)), dim3(256), 0, s, (const float*)dy,
                           (const float*)y, (float*)dres, numel);
    return hipGetLastError();
}

hipError_t launch_l1_grad(int dtype, const void* y, const void* t, void* dy, long long numel, int mask_by_y,
                          hipStream_t s) {
    if (numel <= 0) return hipSuccess;
    const float inv = (float)(1.0 / (double)numel);
    if (dtype == 1)
        SOL_LAUNCH(l1_grad_kernel<true>, dim3(blocks_for((numel + 7) / 8)), dim3(256), 0, s, y, t, dy, numel, inv,
                           mask_by_y);
    else
        SOL_LAUNCH(l1_grad_kernel<false>, dim3(blocks_for(numel)), dim3(256), 0, s, y, t, dy, numel, inv, mask_by_y);
    return hipGetLastError();
}

// bf16, channels % 8 == 0: one thread per (output pixel, 8 channels), 16-byte loads and stores.  Comparing the
// values as floats (bf16 << 16) keeps the result one of the inputs, so no rounding is involved.
// K > 0: the window edge is k = K, known at compile time: all K * K loads are requested before the first comparison
// (at coordinates clamped into the image; a tap outside the image then counts as -inf), one memory round trip per
// thread instead of one per tap.  K == 0: any k, tap by tap.
template <int K>
__global__ __launch_bounds__(256) void maxpool_bf16x8_kernel(const bf16_t* x, bf16_t* y, int N, int H, int W, int C, int k,
                                                             int stride, int pad, int Ho, int Wo) {
    const int c8 = C >> 3;
    const long long total = (long long)N * Ho * Wo * c8;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cc = (int)(idx % c8);
    long long pix = idx / c8;
    const int wo = (int)(pix % Wo);
    pix /= Wo;
    const int ho = (int)(pix % Ho);
    const int n = (int)(pix / Ho);
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = -INFINITY;
    auto take = [&](const uintx4& v, bool inside) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = inside ? __uint_as_float(v[e] << 16) : -INFINITY;
            const float hi2 = inside ? __uint_as_float(v[e] & 0xffff0000u) : -INFINITY;
            m[2 * e] = lo > m[2 * e] ? lo : m[2 * e];
            m[2 * e + 1] = hi2 > m[2 * e + 1] ? hi2 : m[2 * e + 1];
        }
    };
    if constexpr (K > 0) {
        uintx4 v[K * K];
        bool inside[K * K];
#pragma unroll
        for (int kh = 0; kh < K; ++kh)
#pragma unroll
            for (int kw = 0; kw < K; ++kw) {
                const int hi = ho * stride - pad + kh, wi = wo * stride - pad + kw;
                inside[kh * K + kw] = (unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W;
                const int hc = hi < 0 ? 0 : (hi >= H ? H - 1 : hi), wc = wi < 0 ? 0 : (wi >= W ? W - 1 : wi);
                v[kh * K + kw] = *reinterpret_cast<const uintx4*>(x + (((long long)n * H + hc) * W + wc) * C + cc * 8);
            }
#pragma unroll
        for (int t = 0; t < K * K; ++t) take(v[t], inside[t]);
    } else {
        for (int kh = 0; kh < k; ++kh) {
            const int hi = ho * stride - pad + kh;
            if ((unsigned)hi >= (unsigned)H) continue;
            for (int kw = 0; kw < k; ++kw) {
                const int wi = wo * stride - pad + kw;
                if ((unsigned)wi >= (unsigned)W) continue;
                take(*reinterpret_cast<const uintx4*>(x + (((long long)n * H + hi) * W + wi) * C + cc * 8), true);
            }
        }
    }
    uintx4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (__float_as_uint(m[2 * e]) >> 16) | (__float_as_uint(m[2 * e + 1]) & 0xffff0000u);
    store16_through(y + idx * 8, o);
}

hipError_t launch_maxpool(int dtype, const void* x, void* y, int N, int H, int W, int C, int k, int stride, int pad,
                          hipStream_t s) {
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const long long total = (long long)N * Ho * Wo * C;
    if (total <= 0) return hipSuccess;
    if (dtype == 1 && (C & 7) == 0 && k == 3)
        SOL_LAUNCH(maxpool_bf16x8_kernel<3>, dim3(blocks_for(total >> 3)), dim3(256), 0, s, (const bf16_t*)x,
                           (bf16_t*)y, N, H, W, C, k, stride, pad, Ho, Wo);
    else if (dtype == 1 && (C & 7) == 0)
        SOL_LAUNCH(maxpool_bf16x8_kernel<0>, dim3(blocks_for(total >> 3)), dim3(256), 0, s, (const bf16_t*)x,
                           (bf16_t*)y, N, H, W, C, k, stride, pad, Ho, Wo);
    else if (dtype == 1)
        SOL_LAUNCH(maxpool_kernel<true>, dim3(blocks_for(total)), dim3(256), 0, s, x, y, N, H, W, C, k, stride,
                           pad, Ho, Wo);
    else
        SOL_LAUNCH(maxpool_kernel<false>, dim3(blocks_for(total)), dim3(256), 0, s, x, y, N, H, W, C, k,
                           stride, pad, Ho, Wo);
    return hipGetLastError();
}

}  // namespace sol
