// Stand-alone timing model of the slice loop of igemm_fast_kernel<128, 128, 2, 2, 4>, used to tell what the loop is
// bound by: per slice and wave 16 MFMAs 32x32x16 bf16, 16 fragment reads (ds_read_b128) from a ring of four stages,
// 8 asynchronous 16-byte copies into the ring, one vmcnt wait and one workgroup barrier -- the kernel's LDS layout,
// swizzle, fragment addresses and instruction order, with the copy addresses of the 3x3 layer of the benchmark
// bottleneck (pixel rows of 512 bytes, nine taps x four channel slices; weight rows of 4608 bytes shared by all
// workgroups).  Parts can be left out (MFMAs only; MFMAs + fragment reads; everything), and the operands are either
// all zero or random bf16: the instruction stream is the same, the rate is not (the matrix cores' rate on this chip
// depends on the operand values).  The results of the arithmetic are meaningless; every access is in bounds.
//
//   loop_model            operands all zero
//   loop_model --random   random bf16 operands
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <vector>

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
using buffer_rsrc_t = __amdgpu_buffer_rsrc_t;

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

constexpr int kPixBytes = 12544 * 512 + 16384;     // 64 images of 14 x 14 x 256 bf16, plus the reach of the last tap
constexpr int kWBytes = 256 * 4608;                // 256 output channels x (9 taps x 256 channels) bf16
constexpr int kStages = 4, kStage = 256 * 8;       // ring; 16-byte chunks per stage (128 pixel rows + 128 weight rows)

__device__ __forceinline__ int swizzle(int row) { return (row + (row >> 3)) & 7; }

// Pins the order of one step as the kernel does: the fragment reads of the next step first, then the step's copies
// one by one between its four MFMAs.
template <bool READS, bool COPIES, int NCOPIES>
__device__ __forceinline__ void pin_step() {
    if constexpr (READS) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (COPIES && c < NCOPIES) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
}

template <bool READS, bool COPIES>
__global__ __launch_bounds__(256) void loop_model_kernel(const char* src, float* out, int slices, int random_lds) {
    extern __shared__ uintx4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave & 1, wc = wave >> 1;
    for (int i = tid; i < kStages * kStage; i += 256) {
        uintx4 v = {0u, 0u, 0u, 0u};
        if (random_lds) {        // bf16 values of magnitude 0.125 .. 1 with random sign and mantissa
            unsigned x = (unsigned)i * 2654435761u + 12345u;
            for (int e = 0; e < 4; ++e) {
                x = x * 1664525u + 1013904223u;
                v[e] = ((x >> 8) & 0x807f807fu) | 0x3e003e00u | ((x >> 3) & 0x01800180u);
            }
        }
        lds[i] = v;
    }
    __syncthreads();
    const buffer_rsrc_t pix = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src), 0, kPixBytes, 0x00020000);
    const buffer_rsrc_t wts = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src + kPixBytes), 0, kWBytes, 0x00020000);
    const int tile = blockIdx.x % 196;             // 98 pixel tiles x 2 channel tiles
    unsigned voff[8];
    for (int i = 0; i < 8; ++i) {
        const int lrow = 32 * (i & 3) + 8 * wave + (lane >> 3);
        const int cl = (lane & 7) ^ swizzle(lrow);
        voff[i] = i < 4 ? (unsigned)(((tile >> 1) * 128 + lrow) * 512 + cl * 16) : (unsigned)(((tile & 1) * 128 + lrow) * 4608 + cl * 16);
    }
    int wfo[2][4], pfo[2][4];
    for (int ks = 0; ks < 4; ++ks) {
        const int chunk = 2 * ks + (lane >> 5);
        for (int i = 0; i < 2; ++i) {
            const int rw = wc * 64 + i * 32 + (lane & 31), rp = wp * 64 + i * 32 + (lane & 31);
            wfo[i][ks] = 128 * 8 + rw * 8 + (chunk ^ swizzle(rw));
            pfo[i][ks] = rp * 8 + (chunk ^ swizzle(rp));
        }
    }
    floatx16 acc[2][2];
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bf16x8 wf[2][2], pf[2][2];
    for (int b = 0; b < 2; ++b)
        for (int i = 0; i < 2; ++i) {
            wf[b][i] = __builtin_bit_cast(bf16x8, lds[wfo[i][0]]);
            pf[b][i] = __builtin_bit_cast(bf16x8, lds[pfo[i][0]]);
        }
    int q = 0, q_cs = 0, q_tw = 0, q_th = 0;       // slice to request next: weight slice, channel slice, tap
    auto copy = [&](int i, const uintx4* stage_c) {
        if constexpr (COPIES) {
            uintx4* stage = const_cast<uintx4*>(stage_c);
            const unsigned soff = i < 4 ? (unsigned)((q_th * 14 + q_tw) * 512 + q_cs * 128) : (unsigned)(q * 128);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i < 4 ? pix : wts, (__attribute__((address_space(3))) void*)(stage + (32 * (i & 3) + 8 * wave) * 8 + (i >> 2) * 1024),
                                                     16, voff[i], soff, 0, 0);
        }
    };
    auto read = [&](int buf, const uintx4* st, int ks) {
        if constexpr (READS) {
            for (int i = 0; i < 2; ++i) wf[buf][i] = __builtin_bit_cast(bf16x8, st[wfo[i][ks]]);
            for (int j = 0; j < 2; ++j) pf[buf][j] = __builtin_bit_cast(bf16x8, st[pfo[j][ks]]);
        }
    };
    auto multiply = [&](int buf) {
        for (int i = 0; i < 2; ++i)
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], pf[buf][j], acc[i][j], 0, 0, 0);
    };
    auto slice = [&](auto stage_tag) {
        constexpr int S = decltype(stage_tag)::value;
        const uintx4* st = lds + S * kStage;
        const uintx4* next = lds + ((S + 1) % kStages) * kStage;
        const uintx4* ahead = lds + ((S + kStages - 1) % kStages) * kStage;
        read(1, st, 1);
        multiply(0);
        pin_step<READS, COPIES, 0>();
        read(0, st, 2);
        if constexpr (READS) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        if constexpr (COPIES) {
            __builtin_amdgcn_s_waitcnt(0x0f70 | 8);       // vmcnt <= 8: one slice of copies may stay in flight
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        copy(0, ahead);
        copy(1, ahead);
        multiply(1);
        pin_step<false, COPIES, 2>();
        read(1, st, 3);
        copy(2, ahead);
        copy(3, ahead);
        copy(4, ahead);
        multiply(0);
        pin_step<READS, COPIES, 3>();
        read(0, next, 0);
        copy(5, ahead);
        copy(6, ahead);
        copy(7, ahead);
        multiply(1);
        pin_step<READS, COPIES, 3>();
        if (++q == 36) q = 0;
        if (++q_cs == 4) {
            q_cs = 0;
            if (++q_tw == 3) {
                q_tw = 0;
                if (++q_th == 3) q_th = 0;
            }
        }
    };
    for (int kt = 0; kt < slices; kt += 4) {
        slice(std::integral_constant<int, 0>{});
        slice(std::integral_constant<int, 1>{});
        slice(std::integral_constant<int, 2>{});
        slice(std::integral_constant<int, 3>{});
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) s += acc[i][j][0] + acc[i][j][9];
    out[blockIdx.x * 256 + tid] = s + __builtin_bit_cast(float, lds[tid][0]);
}

static int g_random = 0;

// ns per slice over `launches` back-to-back launches of `slices` slices each (slices a multiple of 4)
template <bool READS, bool COPIES>
static double run(const char* src, float* out, int grid, int slices, int launches) {
    const size_t smem = (size_t)kStages * kStage * 16;
    auto kern = loop_model_kernel<READS, COPIES>;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, 0, src, out, 400, g_random);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < launches; ++r) hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, 0, src, out, slices, g_random);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipGetLastError());
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return (double)ms * 1e6 / slices / launches;
}

template <bool READS, bool COPIES>
static void report(const char* what, const char* src, float* out) {
    const double flop_per_slice = 2.0 * 128 * 128 * 64;
    const double steady = run<READS, COPIES>(src, out, 256, 4000, 1);
    const double t36 = run<READS, COPIES>(src, out, 196, 36, 100) * 36, t144 = run<READS, COPIES>(src, out, 196, 144, 100) * 144;
    printf("%-34s 256 workgroups x 4000 slices: %5.0f ns/slice = %4.0f TFLOP/s; 196 workgroups: %5.2f us per launch of 36 slices, %5.2f us of 144, %3.0f ns/slice between\n",
           what, steady, 256.0 * flop_per_slice / steady / 1e3, t36 / 1e3, t144 / 1e3, (t144 - t36) / 108.0);
    fflush(stdout);
}

int main(int argc, char** argv) {
    g_random = argc > 1 && strcmp(argv[1], "--random") == 0;
    const size_t bytes = (size_t)kPixBytes + kWBytes + 4096;
    char* src;
    float* out;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMemset(src, 0, bytes));
    CHECK(hipMalloc(&out, 256 * 256 * sizeof(float)));
    if (g_random) {
        std::vector<unsigned short> h(bytes / 2);
        unsigned x = 12345u;
        for (size_t i = 0; i < h.size(); ++i) {
            x = x * 1664525u + 1013904223u;
            h[i] = (unsigned short)(((x >> 16) & 0x807f) | (0x3e00 + ((x >> 9) & 0x180)));
        }
        CHECK(hipMemcpy(src, h.data(), bytes, hipMemcpyHostToDevice));
    }
    printf("operands: %s\n", g_random ? "random bf16 (magnitude 0.125 .. 1)" : "all zero");
    report<false, false>("MFMAs only", src, out);
    report<true, false>("MFMAs + fragment reads", src, out);
    report<true, true>("MFMAs + reads + copies + barrier", src, out);
    CHECK(hipFree(src));
    CHECK(hipFree(out));
    return 0;
}
