// Shared declarations of the gfx950 kernels: vector types, bf16 helpers, launch parameter
// blocks.  Device code only sees plain structs passed by value; the host planner fills them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sol {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

typedef uint16_t bf16_t;   // storage type of one bfloat16 element

constexpr int kWave = 64;

// ---- bf16 <-> f32 (round to nearest even on the way down) -------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);   // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Per 16-bit lane: all-ones where the bf16 value m is > 0, else zero.  (bf16 > 0  <=>  the pattern
// read as a signed 16-bit integer is > 0; NaNs do not occur in stored activations.)  Two packed
// 16-bit instructions per dword: 0 - m with saturation is negative exactly for m > 0 (the
// saturation keeps -32768, i.e. -0.0, from wrapping to itself), and the arithmetic shift spreads the sign.
__device__ __forceinline__ uintx4 positive_lanes(uintx4 m) {
    const shortx8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const shortx8 neg = __builtin_elementwise_sub_sat(zero, __builtin_bit_cast(shortx8, m));
    return __builtin_bit_cast(uintx4, (shortx8)(neg >> (short)15));
}
__device__ __forceinline__ uintx2 positive_lanes(uintx2 m) {
    const shortx4 zero = {0, 0, 0, 0};
    const shortx4 neg = __builtin_elementwise_sub_sat(zero, __builtin_bit_cast(shortx4, m));
    return __builtin_bit_cast(uintx2, (shortx4)(neg >> (short)15));
}
// Per 16-bit lane: keep v where the bf16 value m is > 0, else +0.
__device__ __forceinline__ uintx4 mask_where_positive(uintx4 v, uintx4 m) { return v & positive_lanes(m); }
__device__ __forceinline__ uintx2 mask_where_positive(uintx2 v, uintx2 m) { return v & positive_lanes(m); }

// ---- asynchronous global -> LDS copies (16 bytes per lane, no register staging) -----------
// The wave's 64 pieces land at lds_wave_base + 16 * lane; lds_wave_base must be wave-uniform.
// Completion is tracked by vmcnt; nothing orders these copies against LDS reads except the
// explicit waits and barriers below.
__device__ __forceinline__ void dma16_to_lds(const void* gsrc, void* lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}
// Same copy through a buffer descriptor: address = base + voff + soff, where soff is wave-uniform
// (an SGPR: no vector instruction is spent on it) and a lane whose offset is >= the descriptor's
// size reads zeros instead of memory.  On gfx950 the range check is on voff + soff without
// wrap-around (measured both ways: an all-ones voff plus any soff reads zeros, and so does an in-range
// voff whose sum with soff passes the end), so a descriptor must span everything soff can reach.
typedef __amdgpu_buffer_rsrc_t buffer_rsrc_t;
__device__ __forceinline__ buffer_rsrc_t make_buffer_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void dma16_buf_to_lds(buffer_rsrc_t rs, unsigned voff, unsigned soff, void* lds_wave_base) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)lds_wave_base, 16, voff,
                                             soff, 0, 0);
}
constexpr unsigned kOutOfRange = 0xffffffffu;    // OR-ed into voff: lane reads zeros

// 16-byte store that writes through the L2 instead of leaving a dirty line there.  A kernel that writes tens of
// megabytes with plain stores pays for their write-back when it ends (all of its dirty lines at once, after the last
// workgroup); written through, the same bytes leave while the kernel still computes.  Readers find the data where
// they found it before (the line stays in L2, clean).
__device__ __forceinline__ void store16_through(void* dst, uintx4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(dst), "v"(v) : "memory");
}

// s_waitcnt with vmcnt = N and lgkmcnt = 0 (expcnt untouched): at most N vector-memory
// operations of this wave still in flight, all of its LDS operations done.
template <int N>
__device__ __forceinline__ void wait_vm_and_lds() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
}
// Workgroup barrier without the memory fence of __syncthreads() (which would wait for every
// outstanding prefetch); callers wait for exactly what they need first.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Forces a launch parameter into a scalar register at this point.  Kernel arguments live in memory and
// the compiler fetches each one where it is first used, waiting for every fetch separately; a kernel
// that names all of its parameters here, at the top, pays one memory round trip for the batch
// instead of one per use site (each costs several hundred nanoseconds on a cold scalar cache).
#ifndef SOL_FETCH_NOW_8
#define SOL_FETCH_NOW_8(a, b, c, d, e, f, g, h) \
    asm volatile("" ::"s"(a), "s"(b), "s"(c), "s"(d), "s"(e), "s"(f), "s"(g), "s"(h))
#endif

// Workgroup ids are dealt round-robin to the 8 XCDs (each with an L2 of its own); this gives every XCD a
// contiguous range of logical tile indices, so that tiles sharing activation rows or a weight panel also
// share an L2.  nblocks = workgroups of the launch that take part.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
    const int per = nblocks >> 3, rem = nblocks & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    const int start = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
    return start + idx;
}

// ---- division by a launch-invariant divisor (n < 2^31): q = (mulhi(n, magic) + n) >> shift ------
struct FastDiv {
    uint32_t magic, shift;
};
inline FastDiv make_fast_div(uint32_t d) {
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    const uint64_t m = ((1ull << 32) * ((1ull << s) - d)) / d + 1;
    return FastDiv{(uint32_t)m, s};
}
__device__ __forceinline__ uint32_t fast_div(uint32_t n, FastDiv d) { return (__umulhi(n, d.magic) + n) >> d.shift; }

// ---- implicit-GEMM launch parameters -----------------------------------------------------
// One "row class" describes which GEMM rows (pixels) a group of workgroups produces and how a
// row and a filter tap map to a source pixel.  The forward pass has one class; the data
// gradient of a stride-s block has s*s classes (input pixels grouped by their residue mod s,
// each with only the taps that can reach it).
struct RowClass {
    int rows;               // GEMM rows of this class = N * Rh * Rw
    int Rh, Rw;             // rows per image
    int h_mul, h_off;       // source row   = rh * h_mul + h_off + th * tap_step
    int w_mul, w_off;       // source col   = rw * w_mul + w_off + tw * tap_step
    int Th, Tw;             // taps of this class
    int tap_step;           // +1 (forward) or -1 (data gradient)
    int oh_mul, oh_off;     // output row   = rh * oh_mul + oh_off
    int ow_mul, ow_off;     // output col   = rw * ow_mul + ow_off
    int tile_begin;         // index of this class' first pixel tile in the launch
    int linear;             // bit 0: source pixel index == row (1x1, stride 1, no padding);
                            // bit 1: output pixel index == row (all rows of the output, in order)
    long long b_off;        // element offset of this class' weight matrix [Nc][Th*Tw*Cs]
    FastDiv div_img, div_rw;// divisors Rh*Rw and Rw (row index -> image, row and column in the image)
};

constexpr int kMaxClasses = 4;

// reduction of the split weight gradient (wgrad.hip, reduce_rows.h)
struct ReduceParams {
    const float* partial;       // [splits][C_out][K]
    const float* dshift_partial;// [splits][C_out]
    const void* W;              // [C_out][K] (bf16 or f32)
    const float* scale;
    float* dW;
    float* dscale;
    float* dshift;
    int C_out, K, splits, accumulate, w_is_bf16;
};

struct IgemmParams {
    const bf16_t* src;          // gathered activation: x (forward) or dy (data gradient)
    const bf16_t* src_mask;     // data gradient with ReLU: the block's y (mask y > 0); else null
    const bf16_t* wmat;         // weight matrices, K-contiguous rows
    bf16_t* out;                // y or dx, [N][Hout][Wout][Nc]
    const float* scale;         // forward epilogue (null in the data gradient)
    const float* shift;
    const bf16_t* addend;       // residual (forward) / dx_addend (data gradient); may be null
    const bf16_t* addend_mask;  // optional gate of the addend (mask value > 0)
    const bf16_t* out_mask;     // optional gate of the stored result (0 where mask value <= 0)
    unsigned src_bytes;         // size of the gathered activation tensor
    int Hs, Ws, Cs;             // source image height, width, channels
    int Nc;                     // GEMM columns = output channels of this GEMM
    int Hout, Wout;             // output image
    int relu;                   // forward: clamp at 0
    int ncls;
    int tiles_c;                // channel tiles per pixel tile
    int total_tiles;
    int panel_groups;           // panel kernel only: workgroups per 128-pixel panel ...
    int panel_tiles;            // ... and 128-channel tiles each of them walks over
    RowClass cls[kMaxClasses];
    // pipelined and panel kernels only: red_blocks > 0 appends that many workgroups to the launch, which finish the
    // split weight gradient of the same block (rows red_block, red_block + red_blocks, ...) instead of multiplying
    ReduceParams red;
    int red_blocks;
};

// LDS read with transpose (16-bit elements): within each group of 16 lanes, the 16 x 8-byte
// pieces the lanes address form a 4 x 16 matrix (4 consecutive lanes = one row of 16 elements);
// lane i of the group receives column i, i.e. element i of each of the 4 rows.
typedef short shortx4_lds __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uintx2 lds_read_tr_b64(const void* lds_addr) {
    const shortx4_lds v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) shortx4_lds*)lds_addr);
    return __builtin_bit_cast(uintx2, v);
}

struct PackParams {            // scale-folded, per-row-class transposed weights for the data gradient
    const bf16_t* W;           // [C_out][KH][KW][C_in]
    const float* scale;
    bf16_t* out;               // per class: [C_in][Th*Tw*C_out]
    int C_in, C_out, KH, KW, stride, pad;
};

// ---- weight-gradient launch parameters ---------------------------------------------------
struct WgradParams {
    const bf16_t* dy;           // [M][C_out]
    const bf16_t* y;            // mask source (null when the block has no ReLU)
    const bf16_t* x;            // [N][H][W][C_in]
    float* partial;             // [splits][C_out][K] fp32
    float* dshift_partial;      // [splits][C_out] fp32
    int N, H, W, C_in, C_out, KH, KW, stride, pad, Ho, Wo;
    int M;                      // N*Ho*Wo
    int K;                      // KH*KW*C_in
    int splits;
    int m_per_split;            // multiple of the reduction tile
    int tiles_k, tiles_c;
    FastDiv div_howo, div_wo;   // divisors Ho*Wo and Wo
    // pipelined kernel only: pack_blocks > 0 appends that many workgroups to the launch, which re-pack the
    // weights for the data gradient of the same block (one 64 x 64 tile each) instead of multiplying
    PackParams pack;
    int pack_blocks;
};


}  // namespace sol
