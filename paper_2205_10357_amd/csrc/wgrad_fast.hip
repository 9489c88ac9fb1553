// Pipelined weight-gradient kernel (channel counts that are multiples of 8, dy already masked).
//
//   G[co][k] = sum_m g[m][co] * A[m][k]        A = im2col(x), k = (kh, kw, ci), ci fastest
//
// Both operands are stored in memory with the reduction index m as the row index, so they go
// global -> LDS exactly as they lie (64 rows of 128 channels each per slice, asynchronous 16-byte
// copies into a ring of NS stages, no register staging, no transposing stores).  The transposition
// an MFMA operand needs -- a lane holds 8 consecutive reduction elements of one channel -- is done
// by the LDS read itself: ds_read_b64_tr_b16 hands every lane one column of a 4 x 16 block.
// 16-byte chunks of a row are XOR-swizzled with 2 * (m & 3) so that the four rows a transposing
// read touches fall into different banks.
//
// Each workgroup owns one 128(k) x 128(co) tile of G for one contiguous range of m and writes it
// as fp32 to the workspace (through LDS, so that rows of the [co][k] partial are written as
// contiguous 512-byte pieces); the reduce kernel adds the ranges in a fixed order.
// dshift[co] = sum_m g[m][co] comes out of the same fragments: the waves that own k rows 0..63
// of k-tile 0 issue one extra MFMA per step with an all-ones operand.
#include <type_traits>

#include "launch.h"
#include "pack_tile.h"
#include <sol_lds_tr.h>

namespace sol {

constexpr int WGF_TILE = 128;                 // tile edge along k and along co
constexpr int WGF_BM = 64;                    // reduction rows per slice
constexpr int WGF_OPER = WGF_BM * 16;         // 16-byte chunks of one operand tile
constexpr int WGF_STAGE = 2 * WGF_OPER;       // chunks per stage (x tile, then g tile)
constexpr int WGF_LDW = WGF_TILE + 4;         // fp32 pitch of the output staging tile

// LINEAR: 1x1, stride 1, no padding (the source pixel of row m is pixel m).  It is a template
// parameter, and the column-sum variant of the loop is chosen once outside it, because every scalar
// branch inside the slice loop costs a pipeline bubble that a single wave per SIMD cannot hide.
template <int NS, bool LINEAR>
__global__ __launch_bounds__(256) void wgrad_fast_kernel(const WgradParams p) {
    HIP_DYNAMIC_SHARED(uintx4, lds)
    constexpr int LPS = 8;                    // async copies per thread and slice (4 x rows + 4 g rows)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: keeps LDS bases scalar
    const int tiles = p.tiles_k * p.tiles_c;
    const int nwg = tiles * p.splits;         // workgroups that multiply; the launch may carry re-pack workgroups after them
    if ((int)blockIdx.x >= nwg) {
        pack_dgrad_weights_tile(p.pack, (int)blockIdx.x - nwg, reinterpret_cast<bf16_t*>(lds));
        return;
    }
    const int bid = xcd_remap(blockIdx.x, nwg);
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tk = t % p.tiles_k, tcn = t / p.tiles_k;
    const int k0 = tk * WGF_TILE, co0 = tcn * WGF_TILE;
    const int m_begin = split * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);
    const int nsl = (m_end - m_begin + WGF_BM - 1) / WGF_BM;

    // ---- copy role: rows 16*i + 4*wave + (lane >> 4) of each operand tile, physical chunk lane & 15.
    // Copies go through buffer descriptors (see dma16_buf_to_lds): the row's byte offset is loop
    // invariant, the slice advance is a scalar, and rows past the end of the range / taps outside
    // the image get an out-of-range offset, i.e. zeros.
    const buffer_rsrc_t x_rs = make_buffer_rsrc(p.x, (unsigned)((long long)p.N * p.H * p.W * p.C_in * 2));
    const buffer_rsrc_t g_rs = make_buffer_rsrc(p.dy, (unsigned)((long long)p.M * p.C_out * 2));
    const int mq = lane >> 4, pc = lane & 15;
    const int cl = pc ^ (2 * mq);             // logical chunk kept at physical chunk pc (m & 3 == mq)
    const int kx = k0 + cl * 8;               // first k of this thread's x chunk
    const bool kx_ok = kx < p.K;
    int kh = 0, kw = 0, ci = 0;
    if (kx_ok) {
        const int tap = kx / p.C_in;
        ci = kx - tap * p.C_in;
        kh = tap / p.KW;
        kw = tap - kh * p.KW;
    }
    const int cg = co0 + cl * 8;              // first channel of this thread's g chunk
    const bool cg_ok = cg < p.C_out;
    const int HoWo = p.Ho * p.Wo;
    const int mrow0 = m_begin + 4 * wave + mq;            // this thread's row in slice 0, copy i adds 16*i
    unsigned xrow[4], grow[4];                             // byte offsets at slice 0 (linear x only)
    int nvalid[4];                                         // slices in which copy i's row is inside [m_begin, m_end)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = mrow0 + 16 * i;
        nvalid[i] = m < m_end ? (m_end - m + WGF_BM - 1) / WGF_BM : 0;
        xrow[i] = kx_ok ? (unsigned)(m * p.C_in + ci) * 2u : kOutOfRange;
        grow[i] = cg_ok ? (unsigned)(m * p.C_out + cg) * 2u : kOutOfRange;
    }

    int q_sl = 0;                             // next slice to request
    auto request_part = [&](int part) {       // part 0,1: x rows 2*part, 2*part+1; part 2,3: g rows
        uintx4* st = lds + (q_sl % NS) * WGF_STAGE;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = (part & 1) * 2 + u;
            const unsigned inval = q_sl < nvalid[i] ? 0u : kOutOfRange;
            if (part < 2) {
                if constexpr (LINEAR) {
                    dma16_buf_to_lds(x_rs, xrow[i] | inval, (unsigned)(q_sl * WGF_BM * p.C_in * 2),
                                     st + (16 * i + 4 * wave) * 16);
                } else {
                    const int m = mrow0 + 16 * i + q_sl * WGF_BM;
                    const int n = (int)fast_div((uint32_t)m, p.div_howo);
                    const int rem = m - n * HoWo;
                    const int ho = (int)fast_div((uint32_t)rem, p.div_wo);
                    const int wo = rem - ho * p.Wo;
                    const int hi = ho * p.stride - p.pad + kh, wi = wo * p.stride - p.pad + kw;
                    const bool ok = kx_ok && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
                    const unsigned off = (unsigned)(((n * p.H + hi) * p.W + wi) * p.C_in + ci) * 2u;
                    dma16_buf_to_lds(x_rs, (ok ? off : kOutOfRange) | inval, 0u, st + (16 * i + 4 * wave) * 16);
                }
            } else {
                dma16_buf_to_lds(g_rs, grow[i] | inval, (unsigned)(q_sl * WGF_BM * p.C_out * 2),
                                 st + WGF_OPER + (16 * i + 4 * wave) * 16);
            }
        }
        if (part == 3) ++q_sl;
    };

    // ---- MFMA role: wave grid 2 (k) x 2 (co), 64 x 64 each = 2 x 2 tiles of 32 x 32 ------------
    const int wk = wave & 1, wcn = wave >> 1;
    const int grp = lane >> 4, j = lane & 15;
    // byte offset (inside an operand tile) of this lane's first transposing read of fragment f:
    // row m = 8*(grp>>1) + (j>>2), channels r .. r+3 with r = base + 32*f + 16*(grp&1) + 4*(j&3)
    int xoff[2], goff[2];
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        const int mrow = 8 * (grp >> 1) + (j >> 2);
        const int rx = wk * 64 + 32 * f + 16 * (grp & 1) + 4 * (j & 3);
        const int rg = wcn * 64 + 32 * f + 16 * (grp & 1) + 4 * (j & 3);
        xoff[f] = mrow * 256 + (((rx >> 3) ^ (2 * (mrow & 3))) << 4) + ((rx >> 2) & 1) * 8;
        goff[f] = mrow * 256 + (((rg >> 3) ^ (2 * (mrow & 3))) << 4) + ((rg >> 2) & 1) * 8;
    }
    const bool do_shift = (tk == 0) && (wk == 0);
    floatx16 acc[2][2], accs[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            acc[a][0][v] = 0.f;
            acc[a][1][v] = 0.f;
            accs[a][v] = 0.f;
        }
    }
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nsl) {
#pragma unroll
            for (int part = 0; part < 4; ++part) request_part(part);
        }

    // Fragments of one 16-deep step: x^T rows (2 tiles) and g^T rows (2 tiles), two 8-byte
    // transposing reads each.  STEP is a compile-time constant so the offsets are immediates.
    struct Frags {
        uintx2 r[8];
    };
    auto issue_frags = [&](Frags& fr, lds_addr_t xbase, auto step_tag) {
        constexpr int O = decltype(step_tag)::value * 4096;
        fr.r[0] = lds_tr_read_issue<O>(xbase + xoff[0]);
        fr.r[1] = lds_tr_read_issue<O + 1024>(xbase + xoff[0]);
        fr.r[2] = lds_tr_read_issue<O>(xbase + xoff[1]);
        fr.r[3] = lds_tr_read_issue<O + 1024>(xbase + xoff[1]);
        fr.r[4] = lds_tr_read_issue<O + WGF_OPER * 16>(xbase + goff[0]);
        fr.r[5] = lds_tr_read_issue<O + WGF_OPER * 16 + 1024>(xbase + goff[0]);
        fr.r[6] = lds_tr_read_issue<O + WGF_OPER * 16>(xbase + goff[1]);
        fr.r[7] = lds_tr_read_issue<O + WGF_OPER * 16 + 1024>(xbase + goff[1]);
    };
    auto frag = [](const Frags& fr, int i) {
        return __builtin_bit_cast(bf16x8, uintx4{fr.r[2 * i][0], fr.r[2 * i][1], fr.r[2 * i + 1][0], fr.r[2 * i + 1][1]});
    };
    auto multiply = [&](Frags& fr, auto newer_tag, auto shift_tag) {   // newer_tag: reads issued after fr's that may stay in flight
        lds_tr_wait<decltype(newer_tag)::value>(fr.r[0], fr.r[1], fr.r[2], fr.r[3], fr.r[4], fr.r[5], fr.r[6], fr.r[7]);
        const bf16x8 x0 = frag(fr, 0), x1 = frag(fr, 1), g0 = frag(fr, 2), g1 = frag(fr, 3);
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, g0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, g1, acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, g0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, g1, acc[1][1], 0, 0, 0);
        if constexpr (decltype(shift_tag)::value) {
            accs[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, g0, accs[0], 0, 0, 0);
            accs[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, g1, accs[1], 0, 0, 0);
        }
    };
    const lds_addr_t lds0 = lds_byte_address(lds);

    // One slice.  Per step: wait for this step's fragments (requested one step earlier), request
    // the next step's, issue a quarter of the copies for the slice NS-1 ahead, multiply.
    auto slice = [&](int sl, auto more_tag, auto shift_tag) {
        constexpr bool MORE = decltype(more_tag)::value;
        const lds_addr_t xbase = lds0 + (lds_addr_t)((sl % NS) * WGF_STAGE * 16);
        Frags fa, fb;
        issue_frags(fa, xbase, std::integral_constant<int, 0>{});
        issue_frags(fb, xbase, std::integral_constant<int, 1>{});
        if constexpr (MORE) request_part(0);
        multiply(fa, std::integral_constant<int, 8>{}, shift_tag);
        issue_frags(fa, xbase, std::integral_constant<int, 2>{});
        if constexpr (MORE) request_part(1);
        multiply(fb, std::integral_constant<int, 8>{}, shift_tag);
        issue_frags(fb, xbase, std::integral_constant<int, 3>{});
        if constexpr (MORE) request_part(2);
        multiply(fa, std::integral_constant<int, 8>{}, shift_tag);
        if constexpr (MORE) request_part(3);
        multiply(fb, std::integral_constant<int, 0>{}, shift_tag);
    };

    auto run = [&](auto shift_tag) {
        int sl = 0;
        for (; sl + NS - 1 < nsl; ++sl) {
            wait_vm_and_lds<(NS - 2) * LPS>();
            wg_barrier();
            slice(sl, std::true_type{}, shift_tag);
        }
        for (; sl < nsl; ++sl) {
            wait_vm_and_lds<0>();
            wg_barrier();
            slice(sl, std::false_type{}, shift_tag);
        }
    };
    if (do_shift) run(std::true_type{});
    else run(std::false_type{});

    // ---- column sums: row 0 of the ones-product = accumulator element 0 of lanes 0..31 ----------
    if (do_shift && lane < 32) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int co = co0 + wcn * 64 + 32 * b + lane;
            if (co < p.C_out) p.dshift_partial[(long long)split * p.C_out + co] = accs[b][0];
        }
    }

    // ---- partial tile through LDS: lane holds channel co (lane & 31) and 4 consecutive k per quad
    float* stg = reinterpret_cast<float*>(lds);
    wait_vm_and_lds<0>();
    wg_barrier();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int col = wcn * 64 + 32 * b + (lane & 31);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int kk = wk * 64 + 32 * a + 8 * q + 4 * (lane >> 5);
                *reinterpret_cast<floatx4*>(stg + col * WGF_LDW + kk) =
                    floatx4{acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
            }
    }
    wait_vm_and_lds<0>();
    wg_barrier();
    float* part = p.partial + (long long)split * p.C_out * p.K;
    const int kq = (tid & 31) * 4, r0 = tid >> 5;
#pragma unroll
    for (int ps = 0; ps < WGF_TILE / 8; ++ps) {
        const int row = r0 + 8 * ps;
        const int co = co0 + row, k = k0 + kq;
        if (co < p.C_out && k < p.K)
            store16_through(part + (long long)co * p.K + k,
                            __builtin_bit_cast(uintx4, *reinterpret_cast<const floatx4*>(stg + row * WGF_LDW + kq)));
    }
}

template <int NS, bool LINEAR>
static hipError_t launch_wgf(const WgradParams& p, hipStream_t stream) {
    const size_t stages = (size_t)NS * WGF_STAGE * 16;
    const size_t epi = (size_t)WGF_TILE * WGF_LDW * 4;
    const size_t smem = stages > epi ? stages : epi;
    auto kern = wgrad_fast_kernel<NS, LINEAR>;
    static std::atomic<size_t> granted{0};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, granted); e != hipSuccess) return e;
    SOL_LAUNCH(kern, dim3(p.tiles_k * p.tiles_c * p.splits + p.pack_blocks), dim3(256), smem, stream, p);
    return hipGetLastError();
}

hipError_t launch_wgrad_fast(const WgradParams& p, int stages, hipStream_t stream) {
    const bool linear = p.KH == 1 && p.KW == 1 && p.stride == 1 && p.pad == 0;
    switch (stages) {
        case 2: return linear ? launch_wgf<2, true>(p, stream) : launch_wgf<2, false>(p, stream);
        case 3: return linear ? launch_wgf<3, true>(p, stream) : launch_wgf<3, false>(p, stream);
        default: return linear ? launch_wgf<4, true>(p, stream) : launch_wgf<4, false>(p, stream);
    }
}

}  // namespace sol
