// Pieces shared by the MFMA kernels that stream their operands global -> LDS by DMA
// (global_load_lds) and keep count of the outstanding operations by hand.
#pragma once
#include <type_traits>

#include "common.h"

namespace bl {

// compile-time loop: f(integral_constant<int, B>), ..., f(integral_constant<int, E-1>)
template <int B, int E, class F>
__device__ inline void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    // gfx9 encoding: vmcnt = {[15:14],[3:0]}, expcnt [6:4] = 7 and lgkmcnt [11:8] = 15 (no wait).
    // The compiler barrier keeps ordinary memory operations on their side of the wait.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ inline void block_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

}  // namespace bl
