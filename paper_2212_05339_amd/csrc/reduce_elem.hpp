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

// Up to kMaxSources gradient arrays (micro-batches, or the contributions of several ranks) summed in one pass.
constexpr int kMaxSources = 4;
struct SrcTable {
    const uint16_t* p[kMaxSources];
};

// Group i (4 elements) of a destination: dst 16-byte aligned, every source 8-byte aligned.  The sources are added
// one after the other, each product and each sum rounded to fp32, exactly as NSRC single-source passes would; all
// loads are issued before the first addition.  Returns what was stored.
template <bool ACC, bool FP16, int NSRC>
__device__ __forceinline__ f32x4 reduce_group(float* __restrict__ dst, const SrcTable& srcs, int64_t i, float scale) {
    f32x4* D = reinterpret_cast<f32x4*>(dst) + i;
    u32x2 g[NSRC];
#pragma unroll
    for (int k = 0; k < NSRC; ++k) g[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(srcs.p[k]) + i);
    f32x4 r;
    if constexpr (ACC) r = __builtin_nontemporal_load(D);
    else r = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int k = 0; k < NSRC; ++k) {
        r.x = reduce_elem<FP16>(r.x, g[k].x & 0xFFFFu, scale);
        r.y = reduce_elem<FP16>(r.y, g[k].x >> 16, scale);
        r.z = reduce_elem<FP16>(r.z, g[k].y & 0xFFFFu, scale);
        r.w = reduce_elem<FP16>(r.w, g[k].y >> 16, scale);
    }
    __builtin_nontemporal_store(r, D);
    return r;
}

}  // namespace elixir
