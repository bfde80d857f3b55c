// Device-side twin of the seeded input generator in gen.py (test/bench harness code).
// It fills caller-owned device buffers with hash-derived values; it contains none of
// the optimizer's arithmetic.  Recipe (must stay in step with gen.py):
//   h = mix64(key + GOLD*(idx+1));  s = sum of h's four 16-bit fields - 131070;
//   x = float(s) * scale;  bf16 output keeps the upper 16 bits of x;
//   if zero_pct > 0 and mix64(h ^ LANE2) % 100 < zero_pct the value is +0.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ float value_at(uint64_t key, int64_t idx, float scale, int zero_pct) {
    const uint64_t h = mix64(key + 0x9E3779B97F4A7C15ull * (uint64_t)(idx + 1));
    const int s = (int)((h & 0xFFFFu) + ((h >> 16) & 0xFFFFu) + ((h >> 32) & 0xFFFFu) + (h >> 48)) - 131070;
    float x = __fmul_rn((float)s, scale);
    if (zero_pct > 0) {
        const uint64_t h2 = mix64(h ^ 0xD6E8FEB86659FD93ull);
        if ((h2 % 100ull) < (uint64_t)zero_pct) x = 0.0f;
    }
    return x;
}

template <bool BF16>
__global__ __launch_bounds__(256) void fill_kernel(void* out, int64_t n, uint64_t key, int64_t idx0,
                                                  float scale, int zero_pct) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float x = value_at(key, idx0 + i, scale, zero_pct);
        if (BF16) ((uint16_t*)out)[i] = (uint16_t)(__float_as_uint(x) >> 16);
        else      ((float*)out)[i] = x;
    }
}

template <bool BF16>
int launch(void* out, int64_t n, uint64_t key, int64_t idx0, float scale, int zero_pct, hipStream_t s) {
    if (n <= 0) return 0;
    if (out == nullptr) return (int)hipErrorInvalidValue;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(fill_kernel<BF16>, dim3((unsigned)blocks), dim3(256), 0, s, out, n, key, idx0, scale, zero_pct);
    return (int)hipGetLastError();
}

}  // namespace

extern "C" int synth_fill_bf16(void* d_out, int64_t n, uint64_t key, int64_t idx0, float scale, int zero_pct, void* stream) {
    return launch<true>(d_out, n, key, idx0, scale, zero_pct, (hipStream_t)stream);
}
extern "C" int synth_fill_f32(void* d_out, int64_t n, uint64_t key, int64_t idx0, float scale, int zero_pct, void* stream) {
    return launch<false>(d_out, n, key, idx0, scale, zero_pct, (hipStream_t)stream);
}
