// Transposing LDS reads issued outside the compiler's wait-count bookkeeping.
//
// The compiler orders every LDS read it knows about behind ALL outstanding asynchronous
// global -> LDS copies (it cannot tell which stage of the ring a read touches), which would
// drain the prefetch queue at every step.  These helpers issue ds_read_b64_tr_b16 as opaque
// instructions; the caller waits explicitly (lds_tr_wait) before using the values, and orders
// reads against the copies with its own vmcnt waits and barriers.
#pragma once

#include "common.h"

namespace sol {

typedef unsigned lds_addr_t;      // byte address inside the workgroup's LDS allocation

__device__ __forceinline__ lds_addr_t lds_byte_address(const void* p) {
    return (lds_addr_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Issue one transposing 8-byte read at addr + OFF (see lds_read_tr_b64 for the lane mapping).
template <int OFF>
__device__ __forceinline__ uintx2 lds_tr_read_issue(lds_addr_t addr) {
    uintx2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// Wait until at most N of this wave's LDS operations are outstanding (they return in order, so
// everything but the N newest has arrived); the operands tie the wait to the values so that no
// use of them can be scheduled above it.
template <int N>
__device__ __forceinline__ void lds_tr_wait(uintx2& a, uintx2& b, uintx2& c, uintx2& d, uintx2& e, uintx2& f,
                                            uintx2& g, uintx2& h) {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit field");
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f), "+v"(g), "+v"(h)
                 : "n"(N));
}

}  // namespace sol
