// Reduction of the split weight gradient, row by row: shared by the stand-alone kernel and by the data-gradient
// launches that carry the reduction along as extra workgroups.
#pragma once
#include "common.h"

namespace sol {

// floats of LDS the row reduction needs (256 split sums + 4 wave sums)
constexpr int kReduceLdsFloats = 260;
// most splits a thread has in flight per chunk; reads of up to this many splits beyond the last are issued (and return 0)
constexpr int kReduceBatch = 16;

// The partial sums are read through a buffer descriptor (out-of-range reads return 0, which is how missing splits and
// chunks beyond the row end are skipped without a branch): K % 4 == 0 for the 16-byte loads, and every offset the
// loads can form must stay below 2^31.
inline bool reduce_rows_ok(const ReduceParams& p) {
    return (p.K & 3) == 0 && p.splits >= 1 && p.C_out >= 1 &&
           ((long long)p.splits + kReduceBatch) * p.C_out * p.K * 4 <= 0x7fffffffLL;
}

// A team of TS threads (TS = 64, 128 or 256; 256 / TS teams in the workgroup) finishes row `co` of the weight
// gradient: fixed-order sum over the splits, dW = scale * G, dscale = <W[co,:], G[co,:]> via wavefront shuffles,
// dshift = sum of the split column sums.  Workgroups `block`, `block + nblocks`, ... take 256 / TS rows each per pass.
// A thread takes 4 consecutive elements at a time, CH such chunks TS * 4 apart, with kReduceBatch splits of each in
// flight.  Whatever CH is, every element adds its splits one after the other (+0 for splits that do not exist) and a
// thread adds its elements to the dscale sum in rising order.  TS < 256 needs K <= 4 TS and splits <= TS, and then
// adds the same numbers in the same order as TS = 256 does.  reduce_rows_ok(p) must hold.  `scratch`:
// kReduceLdsFloats floats of LDS.  All 256 threads must call (barriers inside).
// (A compute unit whose loads miss the L2 moves about 25 GB/s whatever it has in flight beyond this: two rows per
// team at once took as long per byte.)
template <int TS, int CH, int BATCH = kReduceBatch>
__device__ __forceinline__ void reduce_rows_vec(const ReduceParams& p, int block, int nblocks, float* scratch) {
    static_assert(TS == 64 || TS == 128 || TS == 256, "one, two or four waves per row");
    static_assert(BATCH >= 1 && BATCH <= kReduceBatch, "reduce_rows_ok allows for kReduceBatch splits beyond the last");
    constexpr int TEAMS = 256 / TS;
    const int tid = threadIdx.x, team = tid / TS, t = tid % TS;
    const unsigned split_bytes = (unsigned)p.C_out * (unsigned)p.K * 4u;
    const buffer_rsrc_t part_rs = make_buffer_rsrc(p.partial, (unsigned)p.splits * split_bytes);
    constexpr unsigned kNowhere = 0x80000000u;      // beyond the buffer whatever split offset is added
    float* ssum = scratch;            // [256]
    float* wsum = scratch + 256;      // [4]
    for (int co0 = block * TEAMS; co0 < p.C_out; co0 += nblocks * TEAMS) {
        const int co = co0 + team;
        const bool live = co < p.C_out;
        const long long row = (long long)(live ? co : 0) * p.K;
        float dot = 0.f, mine = 0.f;
        if (live) {
            // everything a pass needs is requested before the first wait: the column sums of the splits (every thread
            // fetches its share at once; a single thread walking the splits would pay one memory latency per split),
            // the weights of the chunks, then the partial sums
            const float sc = p.scale[co];
            for (int s2 = t; s2 < p.splits; s2 += TS) mine += p.dshift_partial[(long long)s2 * p.C_out + co];
            for (int k = t * 4; k < p.K; k += TS * 4 * CH) {
                floatx4 g[CH], w[CH];
                unsigned voff[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int kc = k + c * TS * 4;
                    g[c] = floatx4{0.f, 0.f, 0.f, 0.f};
                    w[c] = g[c];
                    voff[c] = kc < p.K ? (unsigned)(row + kc) * 4u : kNowhere;
                    if (kc < p.K) {
                        if (p.w_is_bf16) {
                            const uintx2 wb = *reinterpret_cast<const uintx2*>(reinterpret_cast<const bf16_t*>(p.W) + row + kc);
                            w[c] = floatx4{__uint_as_float(wb[0] << 16), __uint_as_float(wb[0] & 0xffff0000u),
                                           __uint_as_float(wb[1] << 16), __uint_as_float(wb[1] & 0xffff0000u)};
                        } else {
                            w[c] = *reinterpret_cast<const floatx4*>(reinterpret_cast<const float*>(p.W) + row + kc);
                        }
                    }
                }
                for (int s = 0; s < p.splits; s += BATCH) {
                    floatx4 a[CH][BATCH];
#pragma unroll
                    for (int c = 0; c < CH; ++c)
#pragma unroll
                        for (int u = 0; u < BATCH; ++u)
                            a[c][u] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                                      part_rs, voff[c], (unsigned)(s + u) * split_bytes, 0));
#pragma unroll
                    for (int c = 0; c < CH; ++c)
#pragma unroll
                        for (int u = 0; u < BATCH; ++u) g[c] += a[c][u];
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int kc = k + c * TS * 4;
                    if (kc >= p.K) break;
#pragma unroll
                    for (int e = 0; e < 4; ++e) dot = fmaf(w[c][e], g[c][e], dot);
                    floatx4 d = {sc * g[c][0], sc * g[c][1], sc * g[c][2], sc * g[c][3]};
                    if (p.accumulate) d += *reinterpret_cast<const floatx4*>(p.dW + row + kc);
                    store16_through(p.dW + row + kc, __builtin_bit_cast(uintx4, d));
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        if ((tid & 63) == 0) wsum[tid >> 6] = dot;
        ssum[tid] = mine;
        __syncthreads();
        if (live && t == 0) {
            float ds;
            if constexpr (TS == 256) ds = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
            else if constexpr (TS == 128) ds = wsum[2 * team] + wsum[2 * team + 1];
            else ds = wsum[team];
            float db = 0.f;
            const int n = p.splits < TS ? p.splits : TS;
            for (int s2 = 0; s2 < n; ++s2) db += ssum[team * TS + s2];
            p.dscale[co] = p.accumulate ? p.dscale[co] + ds : ds;
            p.dshift[co] = p.accumulate ? p.dshift[co] + db : db;
        }
        __syncthreads();              // the next pass overwrites the sums
    }
}

// Workgroup `block` of `nblocks` that ride along with another kernel's launch: the narrowest team that covers a row,
// up to three chunks per thread at a time where rows are longer than the workgroup.
// SLIM: for host kernels with a small register budget (one chunk, 8 splits in flight).
template <bool SLIM>
__device__ __forceinline__ void reduce_rows_riding(const ReduceParams& p, int block, int nblocks, float* scratch) {
    constexpr int B = SLIM ? 8 : kReduceBatch;
    if (p.K <= 256) reduce_rows_vec<64, 1, B>(p, block, nblocks, scratch);
    else if (p.K <= 512) reduce_rows_vec<128, 1, B>(p, block, nblocks, scratch);
    else if (SLIM || p.K <= 1024) reduce_rows_vec<256, 1, B>(p, block, nblocks, scratch);
    else if (p.K <= 2048) reduce_rows_vec<256, 2, B>(p, block, nblocks, scratch);
    else reduce_rows_vec<256, 3, B>(p, block, nblocks, scratch);
}

// what a launch must satisfy to carry the reduction along (the narrow teams hold one split sum per thread)
inline bool reduce_can_ride(const ReduceParams& p) { return reduce_rows_ok(p) && p.splits <= 64; }

}  // namespace sol
