// fp32 version of the block (SOL_F32): one thread per output element, plain fused
// multiply-adds in fp32.  It exists for the small fp32 correctness configuration (tolerance
// 1e-5, which bf16 operands cannot meet); the throughput path is the bf16 MFMA code.
#include "launch.h"

namespace sol {


__global__ __launch_bounds__(256) void direct_fwd_f32(const DirectParams p) {
    const long long total = (long long)p.N * p.Ho * p.Wo * p.C_out;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int co = (int)(idx % p.C_out);
    long long pix = idx / p.C_out;
    const int wo = (int)(pix % p.Wo);
    pix /= p.Wo;
    const int ho = (int)(pix % p.Ho);
    const int n = (int)(pix / p.Ho);
    float acc = 0.f;
    for (int kh = 0; kh < p.KH; ++kh) {
        const int hi = ho * p.stride - p.pad + kh;
        if ((unsigned)hi >= (unsigned)p.H) continue;
        for (int kw = 0; kw < p.KW; ++kw) {
            const int wi = wo * p.stride - p.pad + kw;
            if ((unsigned)wi >= (unsigned)p.W_) continue;
            const float* xp = p.x + (((long long)n * p.H + hi) * p.W_ + wi) * p.C_in;
            const float* wp = p.W + (((long long)co * p.KH + kh) * p.KW + kw) * p.C_in;
            for (int ci = 0; ci < p.C_in; ++ci) acc = fmaf(xp[ci], wp[ci], acc);
        }
    }
    float v = fmaf(p.scale[co], acc, p.shift[co]);
    if (p.res) v += p.res[idx];
    if (p.relu) v = v > 0.f ? v : 0.f;
    p.y[idx] = v;
}

__global__ __launch_bounds__(256) void direct_dgrad_f32(const DirectParams p) {
    const long long total = (long long)p.N * p.H * p.W_ * p.C_in;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ci = (int)(idx % p.C_in);
    long long pix = idx / p.C_in;
    const int wi = (int)(pix % p.W_);
    pix /= p.W_;
    const int hi = (int)(pix % p.H);
    const int n = (int)(pix / p.H);
    float acc = 0.f;
    for (int kh = 0; kh < p.KH; ++kh) {
        const int th = hi + p.pad - kh;
        if (th < 0 || th % p.stride) continue;
        const int ho = th / p.stride;
        if (ho >= p.Ho) continue;
        for (int kw = 0; kw < p.KW; ++kw) {
            const int tw = wi + p.pad - kw;
            if (tw < 0 || tw % p.stride) continue;
            const int wo = tw / p.stride;
            if (wo >= p.Wo) continue;
            const long long ob = (((long long)n * p.Ho + ho) * p.Wo + wo) * p.C_out;
            for (int co = 0; co < p.C_out; ++co) {
                float g = p.dy[ob + co];
                if (p.ymask && !(p.ymask[ob + co] > 0.f)) g = 0.f;
                acc = fmaf(g * p.scale[co], p.W[(((long long)co * p.KH + kh) * p.KW + kw) * p.C_in + ci], acc);
            }
        }
    }
    if (p.addend) {
        const bool keep = !p.addend_mask || p.addend_mask[idx] > 0.f;
        if (keep) acc += p.addend[idx];
    }
    if (p.dx_mask && !(p.dx_mask[idx] > 0.f)) acc = 0.f;
    p.dx[idx] = acc;
}

// One thread per weight element: unscaled G[co][kh][kw][ci] = sum_m g * x.
__global__ __launch_bounds__(256) void direct_wgrad_f32(const DirectParams p) {
    const int K = p.KH * p.KW * p.C_in;
    const long long total = (long long)p.C_out * K;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ci = (int)(idx % p.C_in);
    long long r = idx / p.C_in;
    const int kw = (int)(r % p.KW);
    r /= p.KW;
    const int kh = (int)(r % p.KH);
    const int co = (int)(r / p.KH);
    float acc = 0.f;
    for (int n = 0; n < p.N; ++n)
        for (int ho = 0; ho < p.Ho; ++ho) {
            const int hi = ho * p.stride - p.pad + kh;
            if ((unsigned)hi >= (unsigned)p.H) continue;
            for (int wo = 0; wo < p.Wo; ++wo) {
                const int wi = wo * p.stride - p.pad + kw;
                if ((unsigned)wi >= (unsigned)p.W_) continue;
                const long long o = (((long long)n * p.Ho + ho) * p.Wo + wo) * p.C_out + co;
                float g = p.dy[o];
                if (p.ymask && !(p.ymask[o] > 0.f)) g = 0.f;
                acc = fmaf(g, p.x[(((long long)n * p.H + hi) * p.W_ + wi) * p.C_in + ci], acc);
            }
        }
    p.G[idx] = acc;
}

// One workgroup per channel: dshift_partial[co] = sum_m g[m][co].
__global__ __launch_bounds__(256) void direct_colsum_f32(const DirectParams p) {
    const int co = blockIdx.x, tid = threadIdx.x;
    const long long M = (long long)p.N * p.Ho * p.Wo;
    float s = 0.f;
    for (long long m = tid; m < M; m += 256) {
        float g = p.dy[m * p.C_out + co];
        if (p.ymask && !(p.ymask[m * p.C_out + co] > 0.f)) g = 0.f;
        s += g;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    __shared__ float wsum[4];
    if ((tid & 63) == 0) wsum[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) p.dshift_partial[co] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

static inline unsigned blocks_for(long long total) { return (unsigned)((total + 255) / 256); }

hipError_t launch_direct_fwd_f32(const DirectParams& p, hipStream_t s) {
    SOL_LAUNCH(direct_fwd_f32, dim3(blocks_for((long long)p.N * p.Ho * p.Wo * p.C_out)), dim3(256), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_direct_dgrad_f32(const DirectParams& p, hipStream_t s) {
    SOL_LAUNCH(direct_dgrad_f32, dim3(blocks_for((long long)p.N * p.H * p.W_ * p.C_in)), dim3(256), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_direct_wgrad_f32(const DirectParams& p, hipStream_t s) {
    SOL_LAUNCH(direct_wgrad_f32, dim3(blocks_for((long long)p.C_out * p.KH * p.KW * p.C_in)), dim3(256), 0, s, p);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    SOL_LAUNCH(direct_colsum_f32, dim3(p.C_out), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace sol
