// elixir_grad_reduce_into_chunk: bf16 gradients summed into the fp32 gradient chunk.
//
//   dst[k] = fl32( (accumulate ? dst[k] : 0) + fl32(scale * widen(src[k])) )
// The multiply and the add are rounded separately (this file is compiled with
// floating-point contraction off), so the result does not depend on whether
// the compiler would have formed a fused multiply-add.
// Traffic per element: 2 bytes read + 4 written, plus 4 read when accumulating.
#include "common.hpp"

using namespace elixir;

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float reduce_elem(float old, uint32_t bf16_bits, float scale) {
    const float t = scale * __uint_as_float(bf16_bits << 16);
    return old + t;
}

constexpr int kUnroll = 4;

// dst 16-byte aligned, src 8-byte aligned; n4 complete groups of 4 elements.
template <bool ACC>
__global__ __launch_bounds__(256) void reduce_vec_kernel(float* __restrict__ dst, const uint16_t* __restrict__ src,
                                                        int64_t n4, float scale) {
    f32x4* D = reinterpret_cast<f32x4*>(dst);
    const u32x2* S = reinterpret_cast<const u32x2*>(src);
    constexpr int64_t kTile = 256 * kUnroll;
    const int64_t n_tiles = (n4 + kTile - 1) / kTile;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t base = tile * kTile + threadIdx.x;
        u32x2 g[kUnroll];
        f32x4 a[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + (int64_t)u * 256;
            if (i < n4) {
                g[u] = __builtin_nontemporal_load(S + i);
                if constexpr (ACC) a[u] = __builtin_nontemporal_load(D + i);
                else a[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + (int64_t)u * 256;
            if (i < n4) {
                f32x4 r;
                r.x = reduce_elem(a[u].x, g[u].x & 0xFFFFu, scale);
                r.y = reduce_elem(a[u].y, g[u].x >> 16, scale);
                r.z = reduce_elem(a[u].z, g[u].y & 0xFFFFu, scale);
                r.w = reduce_elem(a[u].w, g[u].y >> 16, scale);
                __builtin_nontemporal_store(r, D + i);
            }
        }
    }
}

template <bool ACC>
__global__ __launch_bounds__(256) void reduce_scalar_kernel(float* dst, const uint16_t* src, int64_t first, int64_t n,
                                                           float scale) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t k = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride)
        dst[k] = reduce_elem(ACC ? dst[k] : 0.0f, src[k], scale);
}

}  // namespace

extern "C" int elixir_grad_reduce_into_chunk(float* d_grad_chunk, int64_t offset, const uint16_t* d_grad_bf16, int64_t n,
                                             float scale, int accumulate, elixir_stream_t stream) {
    if (n < 0 || offset < 0)
        return fail(ELIXIR_EINVAL, "elixir_grad_reduce_into_chunk: n=%lld, offset=%lld must not be negative",
                    (long long)n, (long long)offset);
    if (n == 0) return ELIXIR_OK;
    if (!d_grad_chunk || !d_grad_bf16) return fail(ELIXIR_EINVAL, "elixir_grad_reduce_into_chunk: NULL pointer");
    if (!aligned(d_grad_chunk, 4) || !aligned(d_grad_bf16, 2))
        return fail(ELIXIR_EALIGN, "elixir_grad_reduce_into_chunk: a pointer is not aligned for its element type");
    hipStream_t s = (hipStream_t)stream;
    float* dst = d_grad_chunk + offset;
    int64_t done = 0;
    if (aligned(dst, 16) && aligned(d_grad_bf16, 8) && n >= 4) {
        const int64_t n4 = n / 4;
        const int64_t tiles = (n4 + 256 * kUnroll - 1) / (256 * kUnroll);
        const unsigned grid = (unsigned)(tiles < 256 * 16 ? tiles : 256 * 16);
        if (accumulate) hipLaunchKernelGGL(reduce_vec_kernel<true>, dim3(grid), dim3(256), 0, s, dst, d_grad_bf16, n4, scale);
        else hipLaunchKernelGGL(reduce_vec_kernel<false>, dim3(grid), dim3(256), 0, s, dst, d_grad_bf16, n4, scale);
        ELIXIR_LAUNCH_CHECK("reduce_vec_kernel");
        done = n4 * 4;
    }
    if (done < n) {
        int64_t blocks = (n - done + 255) / 256;
        if (blocks > 256 * 8) blocks = 256 * 8;
        if (accumulate) hipLaunchKernelGGL(reduce_scalar_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, dst, d_grad_bf16, done, n, scale);
        else hipLaunchKernelGGL(reduce_scalar_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, dst, d_grad_bf16, done, n, scale);
        ELIXIR_LAUNCH_CHECK("reduce_scalar_kernel");
    }
    return ELIXIR_OK;
}
