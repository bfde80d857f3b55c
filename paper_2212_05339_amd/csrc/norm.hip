// elixir_chunk_grad_norm: deterministic global L2 norm of the fp32 gradient chunks
// and the clipping coefficient, both left in device memory.
//
// Stage 1: kNormBlocksPerChunk workgroups per chunk; workgroup b sums, in double
//   precision, the squares of the elements it meets striding through the chunk
//   (a fixed set, whatever the launch): each thread walks its elements in a fixed order, the 64 lanes of a wavefront are combined
//   with a shuffle tree, the 4 wavefronts through LDS in wavefront order.  One
//   double per workgroup goes to a fixed slot of the workspace.
// Stage 2: a single workgroup adds the slots (each thread a fixed strided
//   subset in index order, then the same tree) and writes sqrt(sum) and the
//   clip coefficient.
// No atomics: the tree is a function of (chunk lengths) only, never of timing.
// Traffic: 4 bytes per element.  Double-precision arithmetic (2 ops/element)
// stays far below the fp64 vector rate at HBM speed.
#include "common.hpp"

using namespace elixir;

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxBatch = 128;  // chunks per stage-1 launch (pointer table travels as kernel argument)

struct ChunkTable {
    const float* ptr[kMaxBatch];
    int64_t valid[kMaxBatch];
};

__device__ __forceinline__ double block_sum(double x, double* lds) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < n_waves; ++w) s += lds[w];
    return s;  // valid in thread 0
}

// grid = (kNormBlocksPerChunk, chunks in this batch)
__global__ __launch_bounds__(256) void sumsq_kernel(ChunkTable tab, double* __restrict__ partials) {
    __shared__ double lds[4];
    const int c = blockIdx.y;
    const float* __restrict__ g = tab.ptr[c];
    const int64_t n = tab.valid[c];
    // leading elements up to the first 16-byte boundary, complete groups of 4, trailing elements
    int64_t head = (int64_t)(((16 - (reinterpret_cast<uintptr_t>(g) & 15)) & 15) >> 2);
    if (head > n) head = n;
    const int64_t n4 = (n - head) >> 2;
    const int64_t tail0 = head + (n4 << 2);
    const f32x4* __restrict__ G = reinterpret_cast<const f32x4*>(g + head);

    // Workgroup b takes the 4-element groups b*256 + t, then the same shifted by 1024*256, and so on:
    // at any moment the 1024 workgroups of a chunk read one contiguous window that slides through it.
    constexpr int64_t kStride = (int64_t)kNormBlocksPerChunk * 256;
    double acc = 0.0;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * kStride < n4; i += 4 * kStride) {
        const f32x4 a = __builtin_nontemporal_load(G + i);
        const f32x4 b = __builtin_nontemporal_load(G + i + kStride);
        const f32x4 d = __builtin_nontemporal_load(G + i + 2 * kStride);
        const f32x4 e = __builtin_nontemporal_load(G + i + 3 * kStride);
        acc = fma((double)a.x, (double)a.x, acc); acc = fma((double)a.y, (double)a.y, acc);
        acc = fma((double)a.z, (double)a.z, acc); acc = fma((double)a.w, (double)a.w, acc);
        acc = fma((double)b.x, (double)b.x, acc); acc = fma((double)b.y, (double)b.y, acc);
        acc = fma((double)b.z, (double)b.z, acc); acc = fma((double)b.w, (double)b.w, acc);
        acc = fma((double)d.x, (double)d.x, acc); acc = fma((double)d.y, (double)d.y, acc);
        acc = fma((double)d.z, (double)d.z, acc); acc = fma((double)d.w, (double)d.w, acc);
        acc = fma((double)e.x, (double)e.x, acc); acc = fma((double)e.y, (double)e.y, acc);
        acc = fma((double)e.z, (double)e.z, acc); acc = fma((double)e.w, (double)e.w, acc);
    }
    for (; i < n4; i += kStride) {
        const f32x4 a = __builtin_nontemporal_load(G + i);
        acc = fma((double)a.x, (double)a.x, acc); acc = fma((double)a.y, (double)a.y, acc);
        acc = fma((double)a.z, (double)a.z, acc); acc = fma((double)a.w, (double)a.w, acc);
    }
    if (blockIdx.x == 0) {  // at most 3 leading and 3 trailing elements
        if ((int64_t)threadIdx.x < head) acc = fma((double)g[threadIdx.x], (double)g[threadIdx.x], acc);
        const int64_t k = tail0 + threadIdx.x;
        if (k < n) acc = fma((double)g[k], (double)g[k], acc);
    }
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) partials[(int64_t)c * kNormBlocksPerChunk + blockIdx.x] = s;
}

__global__ __launch_bounds__(1024) void finish_kernel(const double* __restrict__ partials, int64_t n_partials,
                                                     float max_norm, float* d_norm_out, float* d_clip_out) {
    __shared__ double lds[16];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_partials; i += 1024) acc += partials[i];
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const double norm = sqrt(s);
        if (d_norm_out) *d_norm_out = (float)norm;
        if (d_clip_out) {
            double coef = 1.0;
            if (max_norm > 0.0f) {
                const double r = (double)max_norm / (norm + 1e-6);
                coef = r < 1.0 ? r : 1.0;
            }
            *d_clip_out = (float)coef;
        }
    }
}

}  // namespace

extern "C" int elixir_chunk_grad_norm(elixir_ctx* ctx, const float* const* grad_chunks, const int64_t* valid_len,
                                      int n_chunks, float max_norm, float* d_norm_out, float* d_clip_coef_out,
                                      elixir_stream_t stream) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_chunk_grad_norm: ctx is NULL");
    if (n_chunks < 0 || (n_chunks > 0 && (!grad_chunks || !valid_len)))
        return fail(ELIXIR_EINVAL, "elixir_chunk_grad_norm: NULL table or negative n_chunks");
    if (n_chunks > ctx->max_chunks)
        return fail(ELIXIR_ECAP, "elixir_chunk_grad_norm: %d chunks, context sized for %d", n_chunks, ctx->max_chunks);
    if (!aligned(d_norm_out, 4) || !aligned(d_clip_coef_out, 4))
        return fail(ELIXIR_EALIGN, "elixir_chunk_grad_norm: output pointer not 4-byte aligned");
    for (int c = 0; c < n_chunks; ++c) {
        if (valid_len[c] < 0 || valid_len[c] > ctx->max_chunk_elems)
            return fail(valid_len[c] < 0 ? ELIXIR_EINVAL : ELIXIR_ECAP,
                        "elixir_chunk_grad_norm: valid_len[%d]=%lld outside [0, %lld]", c, (long long)valid_len[c],
                        (long long)ctx->max_chunk_elems);
        if (valid_len[c] > 0 && !grad_chunks[c]) return fail(ELIXIR_EINVAL, "elixir_chunk_grad_norm: grad_chunks[%d] is NULL", c);
        if (!aligned(grad_chunks[c], 4)) return fail(ELIXIR_EALIGN, "elixir_chunk_grad_norm: grad_chunks[%d] not 4-byte aligned", c);
    }
    hipStream_t s = (hipStream_t)stream;
    for (int c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const int nb = n_chunks - c0 < kMaxBatch ? n_chunks - c0 : kMaxBatch;
        ChunkTable tab;
        for (int j = 0; j < kMaxBatch; ++j) {
            tab.ptr[j] = j < nb ? grad_chunks[c0 + j] : nullptr;
            tab.valid[j] = j < nb ? valid_len[c0 + j] : 0;
        }
        hipLaunchKernelGGL(sumsq_kernel, dim3(kNormBlocksPerChunk, nb), dim3(256), 0, s, tab,
                           ctx->d_partials + (int64_t)c0 * kNormBlocksPerChunk);
        ELIXIR_LAUNCH_CHECK("sumsq_kernel");
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(1024), 0, s, ctx->d_partials,
                       (int64_t)n_chunks * kNormBlocksPerChunk, max_norm, d_norm_out, d_clip_coef_out);
    ELIXIR_LAUNCH_CHECK("finish_kernel");
    return ELIXIR_OK;
}
