// Fused AdamW kernels for one chunk (gfx950, wave64).
//
// The update is a pure stream: per element 14 bytes are read (bf16 gradient,
// fp32 master, momentum, variance) and 14 written (the three fp32 values and
// the bf16 parameter), nothing is reused, so the kernel is shaped by HBM
// behaviour only.  What measurement on MI355X showed, and what the launch
// shape below encodes:
//   * one workgroup per tile, no grid-stride loop: workgroups are dispatched
//     in index order, so the chip sweeps each of the eight streams as one
//     narrow, sequential front;
//   * the width of that front decides DRAM efficiency.  About 2-3 MB in
//     flight per fp32 stream is the optimum; 128-bit accesses at full
//     occupancy keep 8 MB in flight and lose ~10% of bandwidth to row
//     conflicts.  Hence 64-bit accesses per lane (2 elements per thread,
//     512 contiguous bytes per wavefront instruction), 128-thread workgroups,
//     and a dynamic-LDS reservation that caps residency at 5 wavefronts per
//     SIMD (the LDS itself is not used);
//   * streaming (non-temporal) loads and write-through streaming stores: nothing is read twice.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/elixir_chunk.h"
#include "stream_store.hpp"

namespace elixir {

// Constants of one step, derived on the host in double precision.
struct AdamConsts {
    float lr_wd;         // lr*wd (the decay factor 1 - lr*wd is not representable well enough in fp32)
    float beta1, omb1;   // beta1, 1 - beta1
    float beta2, omb2;   // beta2, 1 - beta2
    float step_size;     // lr / (1 - beta1^t)
    float inv_sqrt_bc2;  // 1 / sqrt(1 - beta2^t)
    float eps;
};

constexpr int kAdamBlock = 128;                 // threads per workgroup of the vector kernel
constexpr int kAdamVec = 2;                     // elements per thread
constexpr unsigned kAdamLdsBytes = 16 * 1024;   // 160 KB / 16 KB = 10 workgroups = 20 wavefronts per CU

__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays a quiet NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// One element, fp32 arithmetic.  Fused multiply-adds only where written; v_sqrt_f32 and
// v_rcp_f32 (1 ulp) instead of the IEEE-exact sequences: the update is ~1e-4 of the weight.
__device__ __forceinline__ void adam_elem(float& p, float& m, float& v, float g, const AdamConsts& c) {
    m = __builtin_fmaf(c.beta1, m, c.omb1 * g);
    v = __builtin_fmaf(c.beta2, v, (c.omb2 * g) * g);
    const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(v), c.inv_sqrt_bc2, c.eps);
    const float upd = (c.step_size * m) * __builtin_amdgcn_rcpf(denom);
    // p*(1 - lr*wd) - upd as p + (-(lr*wd)*p - upd): both small terms are combined first, so p is rounded once
    // and the fp32 rounding of the constant acts on a term of size 1e-6*p, not on p itself
    p = p + __builtin_fmaf(p, -c.lr_wd, -upd);
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Element kinds of the gradient input (GRAD) and of the low-precision parameter copy (OUT).
enum { kF32 = 0, kBF16 = 1, kF16 = 2, kNone = 0 };

// fp16: the hardware conversions (exact widening; round-to-nearest-even narrowing, subnormals kept).
template <int GRAD>
__device__ __forceinline__ void load_grad2(const void* grad, int64_t i, float& g0, float& g1) {
    if constexpr (GRAD == kBF16) {
        const uint32_t gb = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(grad) + i);
        g0 = bf16_bits_to_float(gb & 0xFFFFu);
        g1 = __uint_as_float(gb & 0xFFFF0000u);
    } else if constexpr (GRAD == kF16) {
        const uint32_t gb = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(grad) + i);
        const f16x2 h = __builtin_bit_cast(f16x2, gb);
        g0 = (float)h.x;
        g1 = (float)h.y;
    } else {
        const f32x2 gf = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(grad) + i);
        g0 = gf.x;
        g1 = gf.y;
    }
}

template <int GRAD>
__device__ __forceinline__ float load_grad1(const void* grad, int64_t k) {
    if constexpr (GRAD == kBF16) return bf16_bits_to_float(__builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(grad) + k));
    else if constexpr (GRAD == kF16) return (float)__builtin_bit_cast(_Float16, __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(grad) + k));
    else return __builtin_nontemporal_load(reinterpret_cast<const float*>(grad) + k);
}

template <int OUT>
__device__ __forceinline__ uint32_t lowp_bits(float p) {
    if constexpr (OUT == kF16) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)p);
    else return bf16_rne_bits(p);
}

// The whole update of one pair of elements: shared by the single-chunk and the multi-chunk kernel.
// A wave lives for one pair per lane, so what it waits for before its first memory instruction counts: the loads
// are issued for every lane at once (lanes past the end re-read the last pair instead of branching on n2), and
// the skip flag and the gradient scale are looked at only afterwards, so that all kernel-argument loads can go
// out together instead of one dependent scalar load after the other.
// grad and out may be one and the same array of 16-bit elements (the paper's parameter chunk, which holds the
// gradients after the backward pass, Sec. 4.1): every lane reads its pair before it writes it, and the pair that
// the lanes past the end re-read is never used by them.
template <int GRAD, int OUT>
__device__ __forceinline__ void adam_pair(float* master, float* exp_avg, float* exp_avg_sq, const void* grad, uint16_t* out,
                                          int64_t i_raw, int64_t n2, const AdamConsts& c, const float* d_grad_scale,
                                          const int32_t* d_skip) {
    const bool live = i_raw < n2;
    const int64_t i = live ? i_raw : n2 - 1;
    f32x2* P = reinterpret_cast<f32x2*>(master) + i;
    f32x2* M = reinterpret_cast<f32x2*>(exp_avg) + i;
    f32x2* V = reinterpret_cast<f32x2*>(exp_avg_sq) + i;
    float g0, g1;
    load_grad2<GRAD>(grad, i, g0, g1);
    f32x2 p = __builtin_nontemporal_load(P), m = __builtin_nontemporal_load(M), v = __builtin_nontemporal_load(V);
    if (!live) return;
    if (d_skip && *d_skip) return;
    if (d_grad_scale) {
        const float gs = *d_grad_scale;
        g0 *= gs;
        g1 *= gs;
    }
    float p0 = p.x, m0 = m.x, v0 = v.x, p1 = p.y, m1 = m.y, v1 = v.y;
    adam_elem(p0, m0, v0, g0, c);
    adam_elem(p1, m1, v1, g1, c);
    stream_store(f32x2{p0, p1}, P);
    stream_store(f32x2{m0, m1}, M);
    stream_store(f32x2{v0, v1}, V);
    if constexpr (OUT != kNone)
        stream_store(lowp_bits<OUT>(p0) | (lowp_bits<OUT>(p1) << 16), reinterpret_cast<uint32_t*>(out) + i);
}

// A wave of these kernels lives for one pair per lane, so every round trip it makes before its first vector load
// costs bandwidth.  The single-chunk kernels take what the loads' addresses need (pointers, length) as their first
// arguments, within the 14 dwords that the library's build has the hardware place in scalar registers when a wave
// starts (kernel-argument preloading); the step constants follow and are fetched while the vector loads are in flight.
// The batched kernels index a table by blockIdx.y, which cannot be preloaded: left to itself the compiler fetches the
// length, tests it, and only then fetches the pointers (and later the constants), dependent rounds of scalar loads.
// fetch_together() makes the values it is given live at one point, so their loads are issued back to back and waited
// for once.
template <typename T>
__device__ __forceinline__ void keep_scalar(T v) {
    asm volatile("" ::"s"(v));
}
template <typename... T>
__device__ __forceinline__ void fetch_together(T... v) {
    (keep_scalar(v), ...);
}
__device__ __forceinline__ void fetch_together(const AdamConsts& c) {
    fetch_together(c.lr_wd, c.beta1, c.omb1, c.beta2, c.omb2, c.step_size, c.inv_sqrt_bc2, c.eps);
}

// Vector kernel: thread i owns elements 2i, 2i+1.  Host guarantees 8-byte aligned fp32
// pointers, 4-byte aligned 16-bit pointers, n2 >= 1 complete pairs, gridDim.x * 128 >= n2.
// d_skip (may be NULL): a device flag; when it is non-zero the launch changes nothing (a step
// skipped because of overflowed fp16 gradients).
template <int GRAD, int OUT>
__global__ __launch_bounds__(kAdamBlock) void adam_vec_kernel(float* __restrict__ master, float* __restrict__ exp_avg,
                                                             float* __restrict__ exp_avg_sq,
                                                             const void* grad, uint16_t* out,  // may be the same array
                                                             int64_t n2, const float* __restrict__ d_grad_scale,
                                                             const int32_t* __restrict__ d_skip, AdamConsts c) {
    const int64_t i = (int64_t)blockIdx.x * kAdamBlock + threadIdx.x;
    adam_pair<GRAD, OUT>(master, exp_avg, exp_avg_sq, grad, out, i, n2, c, d_grad_scale, d_skip);
}

// Several chunks in one launch (same step constants for all).  The table travels as a kernel argument.
// grid = (workgroups of the longest chunk, chunks): workgroups are dispatched x-first, so chunk after chunk
// is swept front to back exactly as by adam_vec_kernel, without the drain and refill between launches --
// what makes small chunks launch-bound otherwise.  Workgroups past the end of a shorter chunk exit at once.
constexpr int kAdamMultiMax = 64;
struct AdamMultiTable {
    float* master[kAdamMultiMax];
    float* exp_avg[kAdamMultiMax];
    float* exp_avg_sq[kAdamMultiMax];
    const void* grad[kAdamMultiMax];
    uint16_t* out[kAdamMultiMax];
    int64_t n2[kAdamMultiMax];             // complete pairs per chunk
};

// TILED: tab.master[] holds tiled optimizer chunks (see adam_tiled_kernel below); the two moment tables are unused.
constexpr int64_t kStateTile = ELIXIR_STATE_TILE;
static_assert(kStateTile % (kAdamBlock * kAdamVec) == 0, "a tile must hold whole workgroups");

template <int GRAD, int OUT, bool TILED>
__global__ __launch_bounds__(kAdamBlock) void adam_multi_kernel(AdamMultiTable tab, AdamConsts c,
                                                               const float* __restrict__ d_grad_scale,
                                                               const int32_t* __restrict__ d_skip) {
    const int lo = blockIdx.y;
    const int64_t n2 = tab.n2[lo];
    float* master = tab.master[lo];
    const void* grad = tab.grad[lo];
    uint16_t* out = tab.out[lo];
    fetch_together(n2, master, grad, out, d_grad_scale, d_skip);
    fetch_together(c);
    const int64_t first = (int64_t)blockIdx.x * kAdamBlock;
    if (first >= n2) return;  // a row past the end of a shorter chunk (uniform per workgroup)
    if constexpr (TILED) {
        float* base = master + 2 * kStateTile * (first / (kStateTile / kAdamVec));
        adam_pair<GRAD, OUT>(base, base + kStateTile, base + 2 * kStateTile, grad, out, first + threadIdx.x, n2, c, d_grad_scale, d_skip);
    } else {
        float* exp_avg = tab.exp_avg[lo];
        float* exp_avg_sq = tab.exp_avg_sq[lo];
        fetch_together(exp_avg, exp_avg_sq);
        adam_pair<GRAD, OUT>(master, exp_avg, exp_avg_sq, grad, out, first + threadIdx.x, n2, c, d_grad_scale, d_skip);
    }
}

// Tiled optimizer chunk: master, momentum and variance interleaved in tiles of kStateTile elements,
//   [ p tile | m tile | v tile ] [ p tile | m tile | v tile ] ...
// so that the three fp32 streams of a workgroup sit in one 48 KB stretch instead of three arrays hundreds of MB
// apart.  Measured on MI355X (fresh memory, bf16 and fp32 gradients alike): 85.7-86.5% of the HBM peak against
// 83.3-83.7% for three arrays, for tiles of 2K to 16K elements; one 256-element workgroup per tile is slower than
// three arrays (82.3%).  A tile holds a whole number of workgroups, so the tile of a workgroup is uniform and the
// update itself is adam_pair on shifted base pointers: element e of the chunk is base[e], base[T + e], base[2T + e]
// with base = state + 2 T (e / T).
template <int GRAD, int OUT>
__global__ __launch_bounds__(kAdamBlock) void adam_tiled_kernel(float* __restrict__ state, const void* grad,
                                                               uint16_t* out, int64_t n2,
                                                               const float* __restrict__ d_grad_scale,
                                                               const int32_t* __restrict__ d_skip, AdamConsts c) {
    const int64_t first = (int64_t)blockIdx.x * kAdamBlock;   // first pair of this workgroup
    float* base = state + 2 * kStateTile * (first / (kStateTile / kAdamVec));
    adam_pair<GRAD, OUT>(base, base + kStateTile, base + 2 * kStateTile, grad, out, first + threadIdx.x, n2, c, d_grad_scale, d_skip);
}

// The same two kernels with the step constants read from device memory instead of the kernel arguments: the step
// number is then not part of the launch, so one captured graph can be replayed for step after step (a one-thread
// kernel advances the step counter and derives the constants, see adam.hip).  d_c is uniform: the constants arrive
// through scalar loads that are issued next to the kernel-argument loads and waited for only after the vector loads
// of the update are in flight.
static_assert(sizeof(AdamConsts) == sizeof(((elixir_adam_step_state*)nullptr)->consts), "the step state holds one AdamConsts");

template <int GRAD, int OUT>
__global__ __launch_bounds__(kAdamBlock) void adam_tiled_dev_kernel(float* __restrict__ state, const void* grad, uint16_t* out, int64_t n2,
                                                                   const AdamConsts* __restrict__ d_c,
                                                                   const float* __restrict__ d_grad_scale,
                                                                   const int32_t* __restrict__ d_skip) {
    const AdamConsts c = *d_c;
    const int64_t first = (int64_t)blockIdx.x * kAdamBlock;
    float* base = state + 2 * kStateTile * (first / (kStateTile / kAdamVec));
    adam_pair<GRAD, OUT>(base, base + kStateTile, base + 2 * kStateTile, grad, out, first + threadIdx.x, n2, c, d_grad_scale, d_skip);
}

template <int GRAD, int OUT>
__global__ __launch_bounds__(kAdamBlock) void adam_multi_dev_kernel(AdamMultiTable tab, const AdamConsts* __restrict__ d_c,
                                                                   const float* __restrict__ d_grad_scale,
                                                                   const int32_t* __restrict__ d_skip) {
    const int lo = blockIdx.y;
    const int64_t n2 = tab.n2[lo];
    float* master = tab.master[lo];
    const void* grad = tab.grad[lo];
    uint16_t* out = tab.out[lo];
    fetch_together(n2, master, grad, out, d_c, d_grad_scale, d_skip);
    const int64_t first = (int64_t)blockIdx.x * kAdamBlock;
    if (first >= n2) return;
    const AdamConsts c = *d_c;
    float* base = master + 2 * kStateTile * (first / (kStateTile / kAdamVec));
    adam_pair<GRAD, OUT>(base, base + kStateTile, base + 2 * kStateTile, grad, out, first + threadIdx.x, n2, c, d_grad_scale, d_skip);
}

// Elements [first, n) of a tiled optimizer chunk, one element per thread, any alignment of grad / out.
// d_c (may be NULL): the step constants in device memory, taken instead of c.
template <int GRAD>
__global__ __launch_bounds__(256) void adam_tiled_scalar_kernel(float* state, const void* grad, uint16_t* out, int out_kind,
                                                               int64_t first, int64_t n, AdamConsts c, const AdamConsts* d_c,
                                                               const float* d_grad_scale, const int32_t* d_skip) {
    const int64_t k = first + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    if (d_skip && *d_skip) return;
    if (d_c) c = *d_c;
    float* P = state + k + 2 * kStateTile * (k / kStateTile);
    float g = load_grad1<GRAD>(grad, k);
    float p = P[0], m = P[kStateTile], v = P[2 * kStateTile];
    if (d_grad_scale) g *= *d_grad_scale;
    adam_elem(p, m, v, g, c);
    P[0] = p;
    P[kStateTile] = m;
    P[2 * kStateTile] = v;
    if (out_kind == kBF16) out[k] = (uint16_t)bf16_rne_bits(p);
    else if (out_kind == kF16) out[k] = (uint16_t)lowp_bits<kF16>(p);
}

// Scalar kernel: elements [first, n), any alignment, one element per thread.  Same arithmetic.
// out_kind: kNone / kBF16 / kF16 (run-time: this kernel only sees odd ends and misaligned slices).
template <int GRAD>
__global__ __launch_bounds__(256) void adam_scalar_kernel(float* master, float* exp_avg, float* exp_avg_sq,
                                                         const void* grad, uint16_t* out, int out_kind, int64_t first,
                                                         int64_t n, AdamConsts c, const float* d_grad_scale,
                                                         const int32_t* d_skip) {
    const int64_t k = first + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    if (d_skip && *d_skip) return;
    float g = load_grad1<GRAD>(grad, k);
    float p = __builtin_nontemporal_load(master + k), m = __builtin_nontemporal_load(exp_avg + k),
          v = __builtin_nontemporal_load(exp_avg_sq + k);
    if (d_grad_scale) g *= *d_grad_scale;
    adam_elem(p, m, v, g, c);
    __builtin_nontemporal_store(p, master + k);
    __builtin_nontemporal_store(m, exp_avg + k);
    __builtin_nontemporal_store(v, exp_avg_sq + k);
    if (out_kind == kBF16) __builtin_nontemporal_store((uint16_t)bf16_rne_bits(p), out + k);
    else if (out_kind == kF16) __builtin_nontemporal_store((uint16_t)lowp_bits<kF16>(p), out + k);
}

}  // namespace elixir
