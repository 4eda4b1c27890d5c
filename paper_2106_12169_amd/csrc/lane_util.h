// Small device-side helpers shared by the kernels: compile-time loops and lane writes.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

namespace apnn {

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N-1>)
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

// Lane writes of the two halves of a ballot: reg[lane LA] = low half, reg[lane LB] = high half, other lanes
// unchanged.  The halves come from a vector compare just before; the two wait states this chip needs between a
// vector instruction that writes a scalar register and a vector instruction that reads it are spelled out,
// because the compiler does not look into the statement.
template <int LA, int LB> __device__ __forceinline__ void write_lanes(int &reg, unsigned long long ballot)
{
    const int lo = static_cast<int>(ballot), hi = static_cast<int>(ballot >> 32);
    asm("s_nop 1\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4" : "+v"(reg) : "s"(lo), "s"(hi), "n"(LA), "n"(LB));
}

}  // namespace apnn
