// Small device helpers shared by the gfx950 matrix-core kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace infmllm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr float LOG2E = 1.4426950408889634f;

// A reference maximum is only moved when a row's running maximum has grown by more than this
// (base-2 exponent): exp2(s - ref) then stays below 2^8, well inside bf16/fp32 range, and the
// accumulators are rescaled a handful of times per row instead of once per tile.
constexpr float RESCALE_TAU = 8.0f;

// f(integral_constant<int, I0>) ... f(integral_constant<int, I1 - 1>), in order: a loop whose index is a
// compile-time constant inside the body
template <int I0, int I1, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>{});
        static_for<I0 + 1, I1>(f);
    }
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// the other half-wave's value (lane l <-> lane l ^ 32)
__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32); }

// max of a value and the other half-wave's value, in every lane
__device__ __forceinline__ float xhalf_max(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// sum of a value and the other half-wave's value, in every lane
__device__ __forceinline__ float xhalf_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace infmllm
