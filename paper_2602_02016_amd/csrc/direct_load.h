// Direct global-memory -> LDS loads and explicit wait counts for gfx950 (device code only).
#pragma once
#include <hip/hip_runtime.h>

namespace dash {

// One wavefront-wide direct load: lane l fetches the 16 bytes at base + off (its own choice) and they land at
// lds_dst + 16 l (lane order), no registers in between.  `base` and `lds_dst` must be uniform over the wavefront.
// Written as assembly on purpose: the compiler tracks the direct loads it knows of and, where control flow
// merges, makes LDS reads of OTHER buffers wait for all of them (vmcnt(0) right after a request = the whole
// memory latency exposed).  With this form every wait is explicit: wait_vm_lgkm before the barrier that hands
// the buffer to its readers.  The "memory" clobber keeps LDS accesses on their side of the request.
__device__ __forceinline__ void direct_load16(const char* base, unsigned off, char* lds_dst) {
    const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds), "v"(off), "s"(base)
                 : "memory", "m0");
}

// s_waitcnt: at most N vector-memory operations of this wavefront still in flight (the counter retires them in
// order), and none of its LDS operations (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at "do
// not wait", lgkmcnt 11:8)
template <int N>
__device__ __forceinline__ void wait_vm_lgkm() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
}

}  // namespace dash
