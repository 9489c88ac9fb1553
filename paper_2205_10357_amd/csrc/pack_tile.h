// Re-packing of one 64 x 64 weight tile for the data gradient, shared by the stand-alone kernel and by the
// weight-gradient launch that carries the re-pack along as extra workgroups.
#pragma once
#include "classes.h"
#include "common.h"

namespace sol {

constexpr int kPackTilePitch = 72;     // bf16 elements per LDS row (144 bytes, 16-byte aligned)

// tiles of a weight tensor whose channel counts are multiples of 64
inline bool pack_tiled_ok(const PackParams& p) { return (p.C_in & 63) == 0 && (p.C_out & 63) == 0; }
inline int pack_tile_count(const PackParams& p) { return (int)(((long long)p.C_out * p.KH * p.KW * p.C_in) >> 12); }

// out[class][ci][(jh*Tw + jw)*C_out + co] = bf16(scale[co] * W[co][kh][kw][ci]) for tile b = (tap, 64 co, 64 ci),
// transposed through LDS (tile: 64 * kPackTilePitch elements) so that both the reads (ci contiguous) and the
// writes (co contiguous) are 16-byte pieces of 128-byte rows.  All 256 threads of the workgroup take part.
__device__ __forceinline__ void pack_dgrad_weights_tile(const PackParams& p, int b, bf16_t* tile) {
    constexpr int PITCH = kPackTilePitch;
    const int tid = threadIdx.x;
    const int tiles_ci = p.C_in >> 6, tiles_co = p.C_out >> 6;
    const int tci = b % tiles_ci;
    b /= tiles_ci;
    const int tco = b % tiles_co;
    const int tap = b / tiles_co;
    const int kh = tap / p.KW, kw = tap - kh * p.KW;
    const int co0 = tco * 64, ci0 = tci * 64;
    const int c8 = tid & 7, r0 = tid >> 3;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int co = co0 + r0 + 32 * i;
        const float sc = p.scale[co];
        const uintx4 v = *reinterpret_cast<const uintx4*>(p.W + (((long long)co * p.KH + kh) * p.KW + kw) * p.C_in +
                                                           ci0 + c8 * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t pk = pack_bf16x2(sc * __uint_as_float(v[e] << 16), sc * __uint_as_float(v[e] & 0xffff0000u));
            tile[(c8 * 8 + 2 * e) * PITCH + r0 + 32 * i] = (bf16_t)(pk & 0xffffu);
            tile[(c8 * 8 + 2 * e + 1) * PITCH + r0 + 32 * i] = (bf16_t)(pk >> 16);
        }
    }
    __syncthreads();
    const int s = p.stride;
    const int ph = ((kh - p.pad) % s + s) % s, pw = ((kw - p.pad) % s + s) % s;
    int fh, fw;
    const int Th = class_taps(p.KH, s, p.pad, ph, &fh), Tw = class_taps(p.KW, s, p.pad, pw, &fw);
    const long long off = class_weight_offset(p.C_in, p.C_out, p.KH, p.KW, s, p.pad, ph, pw);
    const int jh = (kh - fh) / s, jw = (kw - fw) / s;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int cil = r0 + 32 * i;
        const uintx4 v = *reinterpret_cast<const uintx4*>(&tile[cil * PITCH + c8 * 8]);
        *reinterpret_cast<uintx4*>(p.out + off + ((long long)(ci0 + cil) * Th * Tw + (jh * Tw + jw)) * p.C_out + co0 +
                                   c8 * 8) = v;
    }
}

}  // namespace sol
