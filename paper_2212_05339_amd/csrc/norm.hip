// elixir_chunk_grad_norm: deterministic global L2 norm of the fp32 gradient chunks
// (elixir_chunk_grad_norm_lp: of 16-bit gradient chunks) and the clipping coefficient,
// both left in device memory.
//
// Stage 1: kNormBlocksPerChunk single-wavefront workgroups per chunk; workgroup b sums, in double
//   precision, the squares of the elements it meets striding through the chunk
//   (a fixed set, whatever the launch): each lane walks its elements in a fixed order into four
//   accumulators that are combined in a fixed order, the 64 lanes with a shuffle tree.  One
//   double per workgroup goes to a fixed slot of the workspace.
// Stage 2: a single workgroup adds the slots (each thread a fixed strided
//   subset in index order, then the same tree) and writes sqrt(sum) and the
//   clip coefficient.
// No atomics: the tree is a function of the chunk lengths and of each chunk pointer's offset from a 16-byte boundary
// (the elements in front of the first boundary are peeled), never of timing or of the launch.
// Traffic: 4 bytes per element.  When the gradients are being written anyway -- the last micro-batch of the
// reduction -- elixir_grad_reduce_chunk_sumsq produces the same per-chunk slots from the values in registers and the
// 4-byte re-read disappears (stage 1b below).  Double-precision arithmetic (2 ops/element)
// stays far below the fp64 vector rate at HBM speed.
#include <mutex>

#include "common.hpp"
#include "reduce_elem.hpp"

using namespace elixir;

namespace {

constexpr int kMaxBatch = 128;  // chunks per stage-1 launch (pointer table travels as kernel argument)

struct ChunkTable {
    const float* ptr[kMaxBatch];
    int64_t valid[kMaxBatch];
};

// Workspace of elixir_chunk_grad_norm_noalloc: the per-chunk partial sums live in this array, which is part of the
// library's code object (one copy per GPU that loads the library, kept until the process ends), so the call needs no
// context and no allocation.  In host code the name below is only a handle: the array's device address is looked up
// once per device (scratch_for_device) and that pointer is what kernels and host calls are given.
constexpr int kNoAllocMaxChunks = 512;                                                          // 512 x 1024 doubles = 4 MiB
static __device__ __align__(256) double scratch[(size_t)kNoAllocMaxChunks * kNormBlocksPerChunk];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on device d, nullptr until looked up

// Device address of `scratch` on the CURRENT device (looked up on first use, with that device current).
int scratch_for_device(const char* what, double** out) {
    int dev = -1;
    ELIXIR_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ELIXIR_ECAP, "%s: device %d, the library keeps workspaces for devices 0..%d", what, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        double* p = nullptr;
        ELIXIR_HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ELIXIR_EHIP, "%s: hipGetSymbolAddress returned a NULL address", what);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ELIXIR_OK;
}

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

// grid = (kNormBlocksPerChunk, chunks in this batch); one wavefront per workgroup.
// Measured on 24 x 64Mi and 24 x 128Mi elements of fresh memory: 1024 single-wavefront workgroups per chunk with
// four 128-bit loads in flight per lane read at 7.0 TB/s; the same kernel with 256-thread workgroups (four times
// the threads per chunk, a window four times as wide) reaches 6.1 / 5.5 TB/s.
constexpr int kSumsqBlock = 64;

__global__ __launch_bounds__(kSumsqBlock) void sumsq_kernel(ChunkTable tab, double* __restrict__ partials) {
    const int c = blockIdx.y;
    const float* __restrict__ g = tab.ptr[c];
    const int64_t n = tab.valid[c];
    // leading elements up to the first 16-byte boundary, complete groups of 4, trailing elements
    int64_t head = (int64_t)(((16 - (reinterpret_cast<uintptr_t>(g) & 15)) & 15) >> 2);
    if (head > n) head = n;
    const int64_t n4 = (n - head) >> 2;
    const int64_t tail0 = head + (n4 << 2);
    const f32x4* __restrict__ G = reinterpret_cast<const f32x4*>(g + head);

    // Workgroup b takes the 4-element groups b*64 + lane, then the same shifted by 1024*64, and so on:
    // at any moment the 1024 workgroups of a chunk read one contiguous window that slides through it.
    // Four accumulators, one per load of an iteration, combined in a fixed order at the end.
    constexpr int64_t kStride = (int64_t)kNormBlocksPerChunk * kSumsqBlock;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    int64_t i = (int64_t)blockIdx.x * kSumsqBlock + threadIdx.x;
    for (; i + 3 * kStride < n4; i += 4 * kStride) {
        const f32x4 a = __builtin_nontemporal_load(G + i);
        const f32x4 b = __builtin_nontemporal_load(G + i + kStride);
        const f32x4 d = __builtin_nontemporal_load(G + i + 2 * kStride);
        const f32x4 e = __builtin_nontemporal_load(G + i + 3 * kStride);
        acc0 = fma((double)a.x, (double)a.x, acc0); acc0 = fma((double)a.y, (double)a.y, acc0);
        acc0 = fma((double)a.z, (double)a.z, acc0); acc0 = fma((double)a.w, (double)a.w, acc0);
        acc1 = fma((double)b.x, (double)b.x, acc1); acc1 = fma((double)b.y, (double)b.y, acc1);
        acc1 = fma((double)b.z, (double)b.z, acc1); acc1 = fma((double)b.w, (double)b.w, acc1);
        acc2 = fma((double)d.x, (double)d.x, acc2); acc2 = fma((double)d.y, (double)d.y, acc2);
        acc2 = fma((double)d.z, (double)d.z, acc2); acc2 = fma((double)d.w, (double)d.w, acc2);
        acc3 = fma((double)e.x, (double)e.x, acc3); acc3 = fma((double)e.y, (double)e.y, acc3);
        acc3 = fma((double)e.z, (double)e.z, acc3); acc3 = fma((double)e.w, (double)e.w, acc3);
    }
    for (; i < n4; i += kStride) {
        const f32x4 a = __builtin_nontemporal_load(G + i);
        acc0 = fma((double)a.x, (double)a.x, acc0); acc0 = fma((double)a.y, (double)a.y, acc0);
        acc0 = fma((double)a.z, (double)a.z, acc0); acc0 = fma((double)a.w, (double)a.w, acc0);
    }
    if (blockIdx.x == 0) {  // at most 3 leading and 3 trailing elements
        if ((int64_t)threadIdx.x < head) acc0 = fma((double)g[threadIdx.x], (double)g[threadIdx.x], acc0);
        const int64_t k = tail0 + threadIdx.x;
        if (k < n) acc0 = fma((double)g[k], (double)g[k], acc0);
    }
    double x = (acc0 + acc1) + (acc2 + acc3);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    if (threadIdx.x == 0) partials[(int64_t)c * kNormBlocksPerChunk + blockIdx.x] = x;
}

// scale: the factor the caller applies to the stored gradients before they count (1 for the fp32 chunks, whose
// reduction has applied it already): the norm is that of scale * g and the coefficient written is scale * clip, the
// factor an update has to apply to the stored gradients.  With scale = 1 both products are exact.
__global__ __launch_bounds__(1024) void finish_kernel(const double* __restrict__ partials, int64_t n_partials,
                                                     float max_norm, double scale, float* d_norm_out, float* d_clip_out) {
    __shared__ double lds[16];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_partials; i += 1024) acc += partials[i];
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const double norm = fabs(scale) * sqrt(s);
        if (d_norm_out) *d_norm_out = (float)norm;
        if (d_clip_out) {
            double coef = 1.0;
            if (max_norm > 0.0f) {
                const double r = (double)max_norm / (norm + 1e-6);
                coef = r < 1.0 ? r : 1.0;
            }
            *d_clip_out = (float)(scale * coef);
        }
    }
}

// Stage 1 for 16-bit gradient chunks (the paper's gradient chunk is a low-precision chunk, Sec. 4.1): the same
// sliding window and the same fixed tree as sumsq_kernel, eight elements per 128-bit load, widened exactly and
// squared and summed in double.  2 bytes per element.
struct LowpChunkTable {
    const uint16_t* ptr[kMaxBatch];
    int64_t valid[kMaxBatch];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool FP16>
__device__ __forceinline__ double sq_pair(uint32_t w, double acc) {
    const double lo = (double)widen<FP16>(w & 0xFFFFu), hi = (double)widen<FP16>(w >> 16);
    return fma(hi, hi, fma(lo, lo, acc));
}

template <bool FP16>
__device__ __forceinline__ double sq_eight(u32x4 a, double acc) {
    return sq_pair<FP16>(a.w, sq_pair<FP16>(a.z, sq_pair<FP16>(a.y, sq_pair<FP16>(a.x, acc))));
}

template <bool FP16>
__global__ __launch_bounds__(kSumsqBlock) void sumsq_lowp_kernel(LowpChunkTable tab, double* __restrict__ partials) {
    const int c = blockIdx.y;
    const uint16_t* __restrict__ g = tab.ptr[c];
    const int64_t n = tab.valid[c];
    // leading elements up to the first 16-byte boundary (at most 7), complete groups of 8, trailing elements (at most 7)
    int64_t head = (int64_t)(((16 - (reinterpret_cast<uintptr_t>(g) & 15)) & 15) >> 1);
    if (head > n) head = n;
    const int64_t n8 = (n - head) >> 3;
    const int64_t tail0 = head + (n8 << 3);
    const u32x4* __restrict__ G = reinterpret_cast<const u32x4*>(g + head);
    constexpr int64_t kStride = (int64_t)kNormBlocksPerChunk * kSumsqBlock;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    int64_t i = (int64_t)blockIdx.x * kSumsqBlock + threadIdx.x;
    for (; i + 3 * kStride < n8; i += 4 * kStride) {
        const u32x4 a = __builtin_nontemporal_load(G + i);
        const u32x4 b = __builtin_nontemporal_load(G + i + kStride);
        const u32x4 d = __builtin_nontemporal_load(G + i + 2 * kStride);
        const u32x4 e = __builtin_nontemporal_load(G + i + 3 * kStride);
        acc0 = sq_eight<FP16>(a, acc0);
        acc1 = sq_eight<FP16>(b, acc1);
        acc2 = sq_eight<FP16>(d, acc2);
        acc3 = sq_eight<FP16>(e, acc3);
    }
    for (; i < n8; i += kStride) acc0 = sq_eight<FP16>(__builtin_nontemporal_load(G + i), acc0);
    if (blockIdx.x == 0) {
        if ((int64_t)threadIdx.x < head) {
            const double x = (double)widen<FP16>(g[threadIdx.x]);
            acc0 = fma(x, x, acc0);
        }
        const int64_t k = tail0 + threadIdx.x;
        if (k < n) {
            const double x = (double)widen<FP16>(g[k]);
            acc0 = fma(x, x, acc0);
        }
    }
    double x = (acc0 + acc1) + (acc2 + acc3);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    if (threadIdx.x == 0) partials[(int64_t)c * kNormBlocksPerChunk + blockIdx.x] = x;
}

// Stage 1b: the gradient reduction of reduce.hip that also leaves the sum of squares of the values it writes, over
// the valid part of the chunk, in stage[blockIdx.x].  One wavefront per workgroup (256 elements): the 64 lanes are
// combined with the fixed shuffle tree alone, no LDS and no barrier, so the pass stays as fast as the plain
// reduction.  Squares and sums are double from the first operation on, as in stage 1 (finite fp32 gradients
// cannot overflow the sum, so a non-finite norm always means a non-finite gradient).  stage[] depends on the
// data only.
constexpr int kFusedBlock = 64;

template <bool ACC, bool FP16, int NSRC>
__global__ __launch_bounds__(kFusedBlock) void reduce_sumsq_kernel(float* __restrict__ dst, const uint16_t* __restrict__ src0, int64_t n4,
                                                                  float scale, const uint16_t* __restrict__ src1,
                                                                  const uint16_t* __restrict__ src2, const uint16_t* __restrict__ src3,
                                                                  int64_t valid, double* __restrict__ stage) {
    // argument order: what the loads need comes first, within the dwords preloaded into scalar registers (see reduce_vec_kernel)
    const int64_t i = (int64_t)blockIdx.x * kFusedBlock + threadIdx.x;
    double x = 0.0;
    if (i < n4) {
        const f32x4 r = reduce_group<ACC, FP16, NSRC>(dst, SrcTable{{src0, src1, src2, src3}}, i, scale);
        const int64_t k = i * 4;
        if (k + 0 < valid) x = fma((double)r.x, (double)r.x, x);
        if (k + 1 < valid) x = fma((double)r.y, (double)r.y, x);
        if (k + 2 < valid) x = fma((double)r.z, (double)r.z, x);
        if (k + 3 < valid) x = fma((double)r.w, (double)r.w, x);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    if (threadIdx.x == 0) stage[blockIdx.x] = x;
}

// The at most 3 elements after the last complete group of 4 (one thread), all sources in order; their squares go to
// the stage entry after the last wavefront's so that the fold below sees them.
template <bool ACC, bool FP16>
__global__ void reduce_sumsq_tail_kernel(float* dst, SrcTable srcs, int n_src, int64_t first, int64_t n, int64_t valid, float scale,
                                         double* stage_slot) {
    double sq = 0.0;
    for (int64_t k = first; k < n; ++k) {
        float r = ACC ? dst[k] : 0.0f;
        for (int j = 0; j < n_src; ++j) r = reduce_elem<FP16>(r, srcs.p[j][k], scale);
        dst[k] = r;
        if (k < valid) sq = fma((double)r, (double)r, sq);
    }
    *stage_slot = sq;
}

// Folds the stage entries of one chunk into its kNormBlocksPerChunk slots: slot j is the sum of the j-th of 1024
// equal contiguous runs of entries, taken by one wavefront (lane l adds entries l, l + 64, ... of the run in order,
// then the fixed shuffle tree).  grid = 256 workgroups of 4 wavefronts.
__global__ __launch_bounds__(256) void fold_stage_kernel(const double* __restrict__ stage, int64_t count, double* __restrict__ slots) {
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t run = (count + kNormBlocksPerChunk - 1) / kNormBlocksPerChunk;
    const int64_t lo = (int64_t)j * run;
    int64_t hi = lo + run;
    if (hi > count) hi = count;
    double acc = 0.0;
    for (int64_t i = lo + lane; i < hi; i += 64) acc += stage[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) slots[j] = acc;
}

// Returns the first launch error (hipSuccess if all three launches were accepted).
template <bool ACC, bool FP16>
hipError_t launch_fused(float* dst, const SrcTable& srcs, int n_src, int64_t n, int64_t valid, float scale, double* stage, double* slots,
                        hipStream_t s) {
    const int64_t n4 = n / 4;
    const int64_t blocks = (n4 + kFusedBlock - 1) / kFusedBlock;  // blocks * 64 threads < 2^32: the caller checked chunk_elems
    if (blocks > 0) {
        const dim3 grid((unsigned)blocks), block(kFusedBlock);
        switch (n_src) {
            case 1: hipLaunchKernelGGL((reduce_sumsq_kernel<ACC, FP16, 1>), grid, block, 0, s, dst, srcs.p[0], n4, scale, srcs.p[1], srcs.p[2], srcs.p[3], valid, stage); break;
            case 2: hipLaunchKernelGGL((reduce_sumsq_kernel<ACC, FP16, 2>), grid, block, 0, s, dst, srcs.p[0], n4, scale, srcs.p[1], srcs.p[2], srcs.p[3], valid, stage); break;
            case 3: hipLaunchKernelGGL((reduce_sumsq_kernel<ACC, FP16, 3>), grid, block, 0, s, dst, srcs.p[0], n4, scale, srcs.p[1], srcs.p[2], srcs.p[3], valid, stage); break;
            default: hipLaunchKernelGGL((reduce_sumsq_kernel<ACC, FP16, 4>), grid, block, 0, s, dst, srcs.p[0], n4, scale, srcs.p[1], srcs.p[2], srcs.p[3], valid, stage); break;
        }
        if (const hipError_t e = hipGetLastError()) return e;
    }
    int64_t count = blocks;
    if (n4 * 4 < n) {
        hipLaunchKernelGGL((reduce_sumsq_tail_kernel<ACC, FP16>), dim3(1), dim3(1), 0, s, dst, srcs, n_src, n4 * 4, n, valid, scale, stage + blocks);
        if (const hipError_t e = hipGetLastError()) return e;
        ++count;
    }
    hipLaunchKernelGGL(fold_stage_kernel, dim3(kNormBlocksPerChunk / 4), dim3(256), 0, s, stage, count, slots);
    return hipGetLastError();
}

}  // namespace

namespace {

// Argument checks and launches shared by elixir_chunk_grad_norm and elixir_chunk_grad_norm_noalloc: the two differ
// only in where the per-chunk partial sums go (max_elems < 0: no limit on a chunk's length).
int norm_fp32_chunks(const char* what, const float* const* grad_chunks, const int64_t* valid_len, int n_chunks,
                     int64_t max_elems, float max_norm, double* partials, float* d_norm_out, float* d_clip_coef_out,
                     hipStream_t s) {
    if (!aligned(d_norm_out, 4) || !aligned(d_clip_coef_out, 4))
        return fail(ELIXIR_EALIGN, "%s: output pointer not 4-byte aligned", what);
    for (int c = 0; c < n_chunks; ++c) {
        if (valid_len[c] < 0 || (max_elems >= 0 && valid_len[c] > max_elems))
            return fail(valid_len[c] < 0 ? ELIXIR_EINVAL : ELIXIR_ECAP, "%s: valid_len[%d]=%lld outside [0, %lld]", what, c,
                        (long long)valid_len[c], (long long)max_elems);
        if (valid_len[c] > 0 && !grad_chunks[c]) return fail(ELIXIR_EINVAL, "%s: grad_chunks[%d] is NULL", what, c);
        if (!aligned(grad_chunks[c], 4)) return fail(ELIXIR_EALIGN, "%s: grad_chunks[%d] not 4-byte aligned", what, c);
    }
    for (int c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const int nb = n_chunks - c0 < kMaxBatch ? n_chunks - c0 : kMaxBatch;
        ChunkTable tab;
        for (int j = 0; j < kMaxBatch; ++j) {
            tab.ptr[j] = j < nb ? grad_chunks[c0 + j] : nullptr;
            tab.valid[j] = j < nb ? valid_len[c0 + j] : 0;
        }
        hipLaunchKernelGGL(sumsq_kernel, dim3(kNormBlocksPerChunk, nb), dim3(kSumsqBlock), 0, s, tab,
                           partials + (int64_t)c0 * kNormBlocksPerChunk);
        ELIXIR_LAUNCH_CHECK("sumsq_kernel");
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(1024), 0, s, partials, (int64_t)n_chunks * kNormBlocksPerChunk, max_norm, 1.0,
                       d_norm_out, d_clip_coef_out);
    ELIXIR_LAUNCH_CHECK("finish_kernel");
    return ELIXIR_OK;
}

}  // namespace

namespace elixir {
// Called by elixir_ctx_create with the context's device current: the address of the static workspace on that device is
// looked up at set-up, so that a later elixir_chunk_grad_norm_noalloc on that device does nothing but launch.
int norm_scratch_init() {
    double* ptr = nullptr;
    return scratch_for_device("elixir_ctx_create", &ptr);
}
}  // namespace elixir

extern "C" int elixir_chunk_grad_norm(elixir_ctx* ctx, const float* const* grad_chunks, const int64_t* valid_len,
                                      int n_chunks, float max_norm, float* d_norm_out, float* d_clip_coef_out,
                                      elixir_stream_t stream) {
    static const char* what = "elixir_chunk_grad_norm";
    if (!ctx) return fail(ELIXIR_EINVAL, "%s: ctx is NULL", what);
    if (n_chunks < 0 || (n_chunks > 0 && (!grad_chunks || !valid_len))) return fail(ELIXIR_EINVAL, "%s: NULL table or negative n_chunks", what);
    if (n_chunks > ctx->max_chunks) return fail(ELIXIR_ECAP, "%s: %d chunks, context sized for %d", what, n_chunks, ctx->max_chunks);
    return norm_fp32_chunks(what, grad_chunks, valid_len, n_chunks, ctx->max_chunk_elems, max_norm, ctx->d_partials, d_norm_out,
                            d_clip_coef_out, (hipStream_t)stream);
}

// The same norm with the partial sums in the library's own static device array: no context, no allocation.
// Every slot the final stage reads is written by the first stage of the same call (a workgroup writes its slot even
// when its chunk is empty), so what an earlier call left in the array never matters and nothing has to be cleared.
extern "C" int elixir_chunk_grad_norm_noalloc(const float* const* grad_chunks, const int64_t* valid_len, int n_chunks,
                                              float max_norm, float* d_norm_out, float* d_clip_coef_out,
                                              elixir_stream_t stream) {
    static const char* what = "elixir_chunk_grad_norm_noalloc";
    if (n_chunks < 0 || (n_chunks > 0 && (!grad_chunks || !valid_len))) return fail(ELIXIR_EINVAL, "%s: NULL table or negative n_chunks", what);
    if (n_chunks > kNoAllocMaxChunks)
        return fail(ELIXIR_ECAP, "%s: %d chunks, the static workspace holds the partial sums of at most %d", what, n_chunks, kNoAllocMaxChunks);
    double* ptr = nullptr;
    if (const int rc = scratch_for_device(what, &ptr)) return rc;
    return norm_fp32_chunks(what, grad_chunks, valid_len, n_chunks, -1, max_norm, ptr, d_norm_out, d_clip_coef_out, (hipStream_t)stream);
}

extern "C" int elixir_chunk_grad_norm_lp(elixir_ctx* ctx, const uint16_t* const* grad_chunks_lowp, int lowp_format,
                                         const int64_t* valid_len, int n_chunks, float scale, float max_norm,
                                         float* d_norm_out, float* d_grad_scale_out, elixir_stream_t stream) {
    static const char* what = "elixir_chunk_grad_norm_lp";
    if (!ctx) return fail(ELIXIR_EINVAL, "%s: ctx is NULL", what);
    if (n_chunks < 0 || (n_chunks > 0 && (!grad_chunks_lowp || !valid_len))) return fail(ELIXIR_EINVAL, "%s: NULL table or negative n_chunks", what);
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (!(fabsf(scale) <= 3.402823466e38f)) return fail(ELIXIR_EINVAL, "%s: scale must be finite", what);
    if (n_chunks > ctx->max_chunks) return fail(ELIXIR_ECAP, "%s: %d chunks, context sized for %d", what, n_chunks, ctx->max_chunks);
    if (!aligned(d_norm_out, 4) || !aligned(d_grad_scale_out, 4)) return fail(ELIXIR_EALIGN, "%s: output pointer not 4-byte aligned", what);
    for (int c = 0; c < n_chunks; ++c) {
        if (valid_len[c] < 0 || valid_len[c] > ctx->max_chunk_elems)
            return fail(valid_len[c] < 0 ? ELIXIR_EINVAL : ELIXIR_ECAP, "%s: valid_len[%d]=%lld outside [0, %lld]", what, c,
                        (long long)valid_len[c], (long long)ctx->max_chunk_elems);
        if (valid_len[c] > 0 && !grad_chunks_lowp[c]) return fail(ELIXIR_EINVAL, "%s: grad_chunks_lowp[%d] is NULL", what, c);
        if (!aligned(grad_chunks_lowp[c], 2)) return fail(ELIXIR_EALIGN, "%s: grad_chunks_lowp[%d] not 2-byte aligned", what, c);
    }
    hipStream_t s = (hipStream_t)stream;
    for (int c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const int nb = n_chunks - c0 < kMaxBatch ? n_chunks - c0 : kMaxBatch;
        LowpChunkTable tab;
        for (int j = 0; j < kMaxBatch; ++j) {
            tab.ptr[j] = j < nb ? grad_chunks_lowp[c0 + j] : nullptr;
            tab.valid[j] = j < nb ? valid_len[c0 + j] : 0;
        }
        double* partials = ctx->d_partials + (int64_t)c0 * kNormBlocksPerChunk;
        if (lowp_format == ELIXIR_LOWP_FP16)
            hipLaunchKernelGGL(sumsq_lowp_kernel<true>, dim3(kNormBlocksPerChunk, nb), dim3(kSumsqBlock), 0, s, tab, partials);
        else
            hipLaunchKernelGGL(sumsq_lowp_kernel<false>, dim3(kNormBlocksPerChunk, nb), dim3(kSumsqBlock), 0, s, tab, partials);
        ELIXIR_LAUNCH_CHECK("sumsq_lowp_kernel");
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(1024), 0, s, ctx->d_partials, (int64_t)n_chunks * kNormBlocksPerChunk, max_norm,
                       (double)scale, d_norm_out, d_grad_scale_out);
    ELIXIR_LAUNCH_CHECK("finish_kernel");
    return ELIXIR_OK;
}

extern "C" int elixir_grad_reduce_sources_chunk_sumsq(elixir_ctx* ctx, int chunk_index, float* d_grad_chunk,
                                                      const uint16_t* const* d_grad_lowp, int n_sources, int lowp_format,
                                                      int64_t chunk_elems, int64_t valid_len, float scale, int accumulate,
                                                      elixir_stream_t stream) {
    static const char* what = "elixir_grad_reduce_sources_chunk_sumsq";
    if (!ctx) return fail(ELIXIR_EINVAL, "%s: ctx is NULL", what);
    if (ctx->fused_open && ctx->fused_stream != stream)
        return fail(ELIXIR_ESTATE, "%s: the calls of one step share the context's workspace and must use one stream (chunk %d arrives on "
                                   "another stream than the calls before it)", what, chunk_index);
    if (chunk_index < 0 || chunk_index >= ctx->max_chunks)
        return fail(ELIXIR_ECAP, "%s: chunk_index=%d, context sized for %d chunks", what, chunk_index, ctx->max_chunks);
    if (chunk_elems < 0 || valid_len < 0 || valid_len > chunk_elems)
        return fail(ELIXIR_EINVAL, "%s: need 0 <= valid_len <= chunk_elems", what);
    if (n_sources < 1) return fail(ELIXIR_EINVAL, "%s: n_sources=%d, at least one gradient array is needed", what, n_sources);
    if (chunk_elems > ctx->max_chunk_elems)
        return fail(ELIXIR_ECAP, "%s: chunk of %lld elements, context sized for %lld", what, (long long)chunk_elems, (long long)ctx->max_chunk_elems);
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (chunk_elems / 4 >= (1ll << 32) - kFusedBlock)  // HIP refuses grids of 2^32 threads or more in x
        return fail(ELIXIR_ECAP, "%s: a chunk of %lld elements does not fit one launch", what, (long long)chunk_elems);
    hipStream_t s = (hipStream_t)stream;
    double* slots = ctx->d_partials + (int64_t)chunk_index * kNormBlocksPerChunk;
    ctx->fused_open = true;
    ctx->fused_stream = stream;
    if (chunk_elems == 0) {  // nothing to reduce: the chunk contributes zero
        hipLaunchKernelGGL(fold_stage_kernel, dim3(kNormBlocksPerChunk / 4), dim3(256), 0, s, ctx->d_stage, (int64_t)0, slots);
        ELIXIR_LAUNCH_CHECK("fold_stage_kernel");
        return ELIXIR_OK;
    }
    if (!d_grad_chunk || !d_grad_lowp) return fail(ELIXIR_EINVAL, "%s: NULL pointer", what);
    if (!aligned(d_grad_chunk, 16)) return fail(ELIXIR_EALIGN, "%s: whole chunks are expected: the fp32 chunk 16-byte aligned", what);
    for (int k = 0; k < n_sources; ++k) {
        if (!d_grad_lowp[k]) return fail(ELIXIR_EINVAL, "%s: gradient array %d is NULL", what, k);
        if (!aligned(d_grad_lowp[k], 8)) return fail(ELIXIR_EALIGN, "%s: whole chunks are expected: the 16-bit gradients 8-byte aligned", what);
    }
    const bool f16 = lowp_format == ELIXIR_LOWP_FP16;
    // all but the last kMaxSources (or fewer) sources go through the plain reduction; the last pass carries the sum of squares
    const int last = (n_sources - 1) / kMaxSources * kMaxSources;
    if (last > 0) {
        const int rc = elixir_grad_reduce_sources_lp(d_grad_chunk, 0, d_grad_lowp, last, lowp_format, chunk_elems, scale, accumulate, stream);
        if (rc != ELIXIR_OK) return rc;
    }
    const int cnt = n_sources - last;
    SrcTable t;
    for (int k = 0; k < kMaxSources; ++k) t.p[k] = k < cnt ? d_grad_lowp[last + k] : nullptr;
    hipError_t e;
    if (accumulate || last > 0) {
        e = f16 ? launch_fused<true, true>(d_grad_chunk, t, cnt, chunk_elems, valid_len, scale, ctx->d_stage, slots, s)
                : launch_fused<true, false>(d_grad_chunk, t, cnt, chunk_elems, valid_len, scale, ctx->d_stage, slots, s);
    } else {
        e = f16 ? launch_fused<false, true>(d_grad_chunk, t, cnt, chunk_elems, valid_len, scale, ctx->d_stage, slots, s)
                : launch_fused<false, false>(d_grad_chunk, t, cnt, chunk_elems, valid_len, scale, ctx->d_stage, slots, s);
    }
    if (e != hipSuccess) return fail(ELIXIR_EHIP, "%s: launch of the fused reduction: %s", what, hipGetErrorString(e));
    return ELIXIR_OK;
}

extern "C" int elixir_grad_reduce_chunk_sumsq(elixir_ctx* ctx, int chunk_index, float* d_grad_chunk, const uint16_t* d_grad_lowp,
                                              int lowp_format, int64_t chunk_elems, int64_t valid_len, float scale,
                                              int accumulate, elixir_stream_t stream) {
    if (chunk_elems > 0 && !d_grad_lowp) return fail(ELIXIR_EINVAL, "elixir_grad_reduce_chunk_sumsq: NULL pointer");
    return elixir_grad_reduce_sources_chunk_sumsq(ctx, chunk_index, d_grad_chunk, &d_grad_lowp, 1, lowp_format, chunk_elems, valid_len,
                                                  scale, accumulate, stream);
}

extern "C" int elixir_chunk_grad_norm_finish(elixir_ctx* ctx, int n_chunks, float max_norm, float* d_norm_out,
                                             float* d_clip_coef_out, elixir_stream_t stream) {
    static const char* what = "elixir_chunk_grad_norm_finish";
    if (!ctx) return fail(ELIXIR_EINVAL, "%s: ctx is NULL", what);
    if (n_chunks < 0) return fail(ELIXIR_EINVAL, "%s: n_chunks is negative", what);
    if (n_chunks > ctx->max_chunks) return fail(ELIXIR_ECAP, "%s: %d chunks, context sized for %d", what, n_chunks, ctx->max_chunks);
    if (!aligned(d_norm_out, 4) || !aligned(d_clip_coef_out, 4)) return fail(ELIXIR_EALIGN, "%s: output pointer not 4-byte aligned", what);
    if (ctx->fused_open && ctx->fused_stream != stream)
        return fail(ELIXIR_ESTATE, "%s: called on another stream than the reductions whose sums it is to fold", what);
    ctx->fused_open = false;
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, ctx->d_partials,
                       (int64_t)n_chunks * kNormBlocksPerChunk, max_norm, 1.0, d_norm_out, d_clip_coef_out);
    ELIXIR_LAUNCH_CHECK("finish_kernel");
    return ELIXIR_OK;
}
