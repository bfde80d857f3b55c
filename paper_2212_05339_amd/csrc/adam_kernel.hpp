// Fused AdamW kernels for one chunk (gfx950, wave64).
//
// The update is a pure stream: per element 14 bytes are read (bf16 gradient,
// fp32 master, momentum, variance) and 14 written (the three fp32 values and
// the bf16 parameter), nothing is reused, so the kernel is organised around
// HBM traffic only:
//   * every memory instruction of a wavefront covers one contiguous span
//     (64 lanes x 16 bytes for fp32, 64 x 8 bytes for bf16);
//   * each thread keeps UNROLL independent groups of 4 elements in flight so
//     that all loads of a tile are issued before the first arithmetic;
//   * a workgroup walks tiles of kBlock*4*UNROLL elements with a grid stride.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elixir {

// Constants of one step, derived on the host in double precision.
struct AdamConsts {
    float decay;         // 1 - lr*wd
    float beta1, omb1;   // beta1, 1 - beta1
    float beta2, omb2;   // beta2, 1 - beta2
    float step_size;     // lr / (1 - beta1^t)
    float inv_sqrt_bc2;  // 1 / sqrt(1 - beta2^t)
    float eps;
};

__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays a quiet NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// One element.  p, m, v are updated in place; returns nothing.
__device__ __forceinline__ void adam_elem(float& p, float& m, float& v, float g, const AdamConsts& c) {
    m = __builtin_fmaf(c.beta1, m, c.omb1 * g);
    v = __builtin_fmaf(c.beta2, v, (c.omb2 * g) * g);
    const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(v), c.inv_sqrt_bc2, c.eps);
    const float upd = (c.step_size * m) * __builtin_amdgcn_rcpf(denom);
    p = __builtin_fmaf(p, c.decay, -upd);
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T x) {
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Vector kernel.  Requirements checked by the host: all pointers 16-byte aligned
// (the bf16 ones 8-byte), n4 = number of complete 4-element groups.
// GRAD_BF16: gradient is bf16 (else fp32).  HAS_OUT: write the bf16 parameter copy.
template <bool GRAD_BF16, bool HAS_OUT, int UNROLL, bool NT_LOAD, bool NT_STORE>
__global__ __launch_bounds__(256) void adam_vec_kernel(float* __restrict__ master, float* __restrict__ exp_avg,
                                                      float* __restrict__ exp_avg_sq, const void* __restrict__ grad,
                                                      uint16_t* __restrict__ out, int64_t n4, AdamConsts c,
                                                      const float* __restrict__ d_grad_scale) {
    const float gs = d_grad_scale ? *d_grad_scale : 1.0f;
    f32x4* P = reinterpret_cast<f32x4*>(master);
    f32x4* M = reinterpret_cast<f32x4*>(exp_avg);
    f32x4* V = reinterpret_cast<f32x4*>(exp_avg_sq);
    const f32x4* G32 = reinterpret_cast<const f32x4*>(grad);
    const u32x2* G16 = reinterpret_cast<const u32x2*>(grad);
    u32x2* O = reinterpret_cast<u32x2*>(out);

    constexpr int64_t kTile = 256 * UNROLL;  // groups per tile
    const int64_t n_tiles = (n4 + kTile - 1) / kTile;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t base = tile * kTile + threadIdx.x;
        f32x4 p[UNROLL], m[UNROLL], v[UNROLL], g[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * 256;
            if (i < n4) {
                if constexpr (GRAD_BF16) {
                    const u32x2 gb = ld<NT_LOAD>(G16 + i);
                    g[u].x = bf16_bits_to_float(gb.x & 0xFFFFu);
                    g[u].y = __uint_as_float(gb.x & 0xFFFF0000u);
                    g[u].z = bf16_bits_to_float(gb.y & 0xFFFFu);
                    g[u].w = __uint_as_float(gb.y & 0xFFFF0000u);
                } else {
                    g[u] = ld<NT_LOAD>(G32 + i);
                }
                p[u] = ld<NT_LOAD>(P + i);
                m[u] = ld<NT_LOAD>(M + i);
                v[u] = ld<NT_LOAD>(V + i);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * 256;
            if (i < n4) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float pe = p[u][e], me = m[u][e], ve = v[u][e];
                    adam_elem(pe, me, ve, gs * g[u][e], c);
                    p[u][e] = pe;
                    m[u][e] = me;
                    v[u][e] = ve;
                }
                st<NT_STORE>(P + i, p[u]);
                st<NT_STORE>(M + i, m[u]);
                st<NT_STORE>(V + i, v[u]);
                if constexpr (HAS_OUT) {
                    u32x2 o;
                    o.x = bf16_rne_bits(p[u].x) | (bf16_rne_bits(p[u].y) << 16);
                    o.y = bf16_rne_bits(p[u].z) | (bf16_rne_bits(p[u].w) << 16);
                    st<NT_STORE>(O + i, o);
                }
            }
        }
    }
}

// Scalar kernel: any alignment, any n.  Same arithmetic, one element per thread per iteration.
template <bool GRAD_BF16>
__global__ __launch_bounds__(256) void adam_scalar_kernel(float* master, float* exp_avg, float* exp_avg_sq,
                                                         const void* grad, uint16_t* out, int64_t first, int64_t n,
                                                         AdamConsts c, const float* d_grad_scale) {
    const float gs = d_grad_scale ? *d_grad_scale : 1.0f;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t k = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) {
        float g;
        if constexpr (GRAD_BF16) g = bf16_bits_to_float(reinterpret_cast<const uint16_t*>(grad)[k]);
        else g = reinterpret_cast<const float*>(grad)[k];
        float p = master[k], m = exp_avg[k], v = exp_avg_sq[k];
        adam_elem(p, m, v, gs * g, c);
        master[k] = p;
        exp_avg[k] = m;
        exp_avg_sq[k] = v;
        if (out) out[k] = (uint16_t)bf16_rne_bits(p);
    }
}

}  // namespace elixir
