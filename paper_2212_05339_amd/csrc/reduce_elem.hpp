// Per-element arithmetic of the gradient reduction, shared by the plain pass (reduce.hip) and the pass that also
// sums squares for the global norm (norm.hip).  Files that include this must be compiled with floating-point
// contraction off: the multiply and the add are rounded separately.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elixir {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// 16 gradient bits -> fp32: bf16 is the upper half of an fp32 pattern; fp16 takes the hardware conversion (exact).
template <bool FP16>
__device__ __forceinline__ float widen(uint32_t bits16) {
    if constexpr (FP16) return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
    else return __uint_as_float(bits16 << 16);
}

template <bool FP16>
__device__ __forceinline__ float reduce_elem(float old, uint32_t bits16, float scale) {
    const float t = scale * widen<FP16>(bits16);
    return old + t;
}

}  // namespace elixir
