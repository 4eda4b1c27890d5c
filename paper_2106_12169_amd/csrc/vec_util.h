// Small vector helpers shared by the kernels: 1-, 2- and 4-word loader vectors.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace apnn {

template <int VW> struct VecT;
template <> struct VecT<4> { using type = uint4; };
template <> struct VecT<2> { using type = uint2; };
template <> struct VecT<1> { using type = uint32_t; };

template <int VW> __device__ __forceinline__ typename VecT<VW>::type vec_zero();
template <> __device__ __forceinline__ uint4 vec_zero<4>() { return make_uint4(0, 0, 0, 0); }
template <> __device__ __forceinline__ uint2 vec_zero<2>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint32_t vec_zero<1>() { return 0u; }

template <int VW> __device__ __forceinline__ typename VecT<VW>::type vec_ones();
template <> __device__ __forceinline__ uint4 vec_ones<4>() { return make_uint4(~0u, ~0u, ~0u, ~0u); }
template <> __device__ __forceinline__ uint2 vec_ones<2>() { return make_uint2(~0u, ~0u); }
template <> __device__ __forceinline__ uint32_t vec_ones<1>() { return ~0u; }

__device__ __forceinline__ int vec_popc(uint4 v) { return __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w); }
__device__ __forceinline__ int vec_popc(uint2 v) { return __popc(v.x) + __popc(v.y); }
__device__ __forceinline__ int vec_popc(uint32_t v) { return __popc(v); }

}  // namespace apnn
