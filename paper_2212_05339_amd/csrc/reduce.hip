// elixir_grad_reduce_into_chunk: bf16 gradients summed into the fp32 gradient chunk.
//
//   dst[k] = fl32( (accumulate ? dst[k] : 0) + fl32(scale * widen(src[k])) )
// The multiply and the add are rounded separately (this file is compiled with
// floating-point contraction off), so the result does not depend on whether
// the compiler would have formed a fused multiply-add.
// Traffic per element: 2 bytes read + 4 written, plus 4 read when accumulating.
#include "common.hpp"
#include "reduce_elem.hpp"
#include "row_plan.hpp"

using namespace elixir;

namespace {

static_assert(kMaxSources == 4, "reduce_vec_kernel names its sources one by one");
constexpr int kVecBlock = 64;   // one 4-element group per thread, one single-wavefront workgroup per 256 elements, no
                                // loop: workgroups are dispatched in index order, so the streams advance as sequential
                                // fronts, with 128-bit accesses at full residency.  Measured on 64Mi elements, 64 / 128 /
                                // 256 threads per workgroup: overwrite 82.8 / 81.0 / 80.3%, accumulate 83.7 / 83.1 / 80.7%
                                // of the HBM peak
// HIP refuses a launch whose grid spans 2^32 threads or more in x: single launches are cut below that, and a row of a
// batched launch is at most kMaxRowTiles workgroups long (longer tensors become several rows)
constexpr int64_t kMaxBlocksPerLaunch = ((1ll << 32) - 1) / 256;
constexpr int64_t kMaxRowTiles = 1ll << 22;

// n4 complete groups of 4 elements, one per thread; NSRC gradient arrays in one pass.  Plain pointer arguments, what
// every pass needs first: the build has the first 14 dwords of a kernel's arguments placed in scalar registers when a
// wave starts (kernel-argument preloading, which does not reach into a table passed by value), so these short-lived
// waves issue their vector loads without waiting for a scalar load.
template <bool ACC, bool FP16, int NSRC>
__global__ __launch_bounds__(kVecBlock) void reduce_vec_kernel(float* __restrict__ dst, const uint16_t* __restrict__ src0, int64_t n4,
                                                              float scale, const uint16_t* __restrict__ src1,
                                                              const uint16_t* __restrict__ src2, const uint16_t* __restrict__ src3,
                                                              int phase) {
    // phase: groups by which dst lies past a KiB boundary; the first workgroup leaves that many lanes idle, so that every
    // wavefront writes one aligned KiB (see row_plan.hpp: 3-5% of the bandwidth on slices in the middle of a chunk)
    const int64_t i = (int64_t)blockIdx.x * kVecBlock + threadIdx.x - phase;
    if (i >= 0 && i < n4) (void)reduce_group<ACC, FP16, NSRC>(dst, SrcTable{{src0, src1, src2, src3}}, i, scale);
}

// elements [first, n), any alignment
template <bool ACC, bool FP16>
__global__ __launch_bounds__(256) void reduce_scalar_kernel(float* dst, const uint16_t* src, int64_t first, int64_t n,
                                                           float scale) {
    const int64_t k = first + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) dst[k] = reduce_elem<FP16>(ACC ? dst[k] : 0.0f, src[k], scale);
}

// Many tensors in one launch.  Gradients arrive tensor by tensor, and most tensors of a transformer are small
// (biases, norms): one launch each leaves the chip idle between launches (the 580 tensors of the 1.5B set take
// 2.6 ms that way, against 1.4 ms of memory time).  grid = (row length, rows): a row is a piece of one tensor
// (row_plan.hpp cuts the tensors into equal pieces plus a tail each and groups rows of similar length), workgroups
// are dispatched x-first, so piece after piece is swept front to back exactly as by reduce_vec_kernel; workgroups
// past the end of a shorter row exit at once.  The table is a kernel argument and blockIdx.y indexes it directly: a
// wave's kernel-argument loads all go out together.  The table is compact (row_plan.hpp), 336 rows to a launch: on the
// tensor list of the 1.5B set that measures like 160 rows, on lists of many small tensors it saves launches (6288
// tensors of 256,000 elements: 77.0% -> 79.5% of the HBM peak).  (Numbering the tiles of all tensors consecutively and
// searching the table for the owner of a tile costs each of these short-lived waves ~200 scalar instructions or a
// chain of dependent loads; measured, it was no faster than one launch per tensor.)
constexpr int kMultiBlock = 64;       // single-wavefront workgroups, as in reduce_vec_kernel

// Rows in the compact form of row_plan.hpp (two bases per launch, 32-bit offsets in groups of 4 elements): 336 rows per
// launch, so the 611 pieces and 383 small tensors of the 1.5B set take four launches.
template <bool ACC, bool FP16>
__global__ __launch_bounds__(kMultiBlock) void reduce_rows_kernel(CompactRows tab, float scale) {
    const int r = blockIdx.y;
    // A wave lives for one group per lane, so what it waits for before its first memory instruction counts: the row's
    // three table entries, the bases and the scale are fetched together, ahead of the test (left to itself the
    // compiler fetches the length, tests, fetches the source, loads, fetches the destination: three round trips
    // instead of one).
    const uint32_t d_off = tab.dst_off[r], s_off = tab.src_off[r], n4 = tab.count[r];
    float* dst_base = reinterpret_cast<float*>(tab.dst_base);
    const uint16_t* src_base = reinterpret_cast<const uint16_t*>(tab.src_base);
    asm volatile("" ::"s"(d_off), "s"(s_off), "s"(n4), "s"(dst_base), "s"(src_base), "s"(scale));
    const uint32_t phase = d_off % kMultiBlock;  // dst_base is KiB-aligned: the row starts this many groups past a KiB boundary
    if (blockIdx.x * kMultiBlock >= n4 + phase) return;  // a row past the end of a shorter piece (uniform per workgroup)
    const int32_t i = (int32_t)(blockIdx.x * kMultiBlock + threadIdx.x) - (int32_t)phase;  // the first workgroup's first lanes idle
    if (i >= 0 && (uint32_t)i < n4)
        (void)reduce_group<ACC, FP16, 1>(dst_base + (int64_t)d_off * 4, SrcTable{{src_base + (int64_t)s_off * 4}}, i, scale);
}

// The vector part of a pass over NSRC sources: n4 groups of 4 elements starting at dst / srcs.
template <bool ACC, bool FP16, int NSRC>
void launch_vec(float* dst, const SrcTable& srcs, int64_t n4, float scale, hipStream_t s) {
    int64_t at = 0;
    while (at < n4) {
        const int64_t phase = row_phase<16, kVecBlock>(dst + at * 4);
        int64_t blocks = (n4 - at + phase + kVecBlock - 1) / kVecBlock;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t cnt = n4 - at < blocks * kVecBlock - phase ? n4 - at : blocks * kVecBlock - phase;
        SrcTable t;
        for (int k = 0; k < kMaxSources; ++k) t.p[k] = k < NSRC ? srcs.p[k] + at * 4 : nullptr;
        hipLaunchKernelGGL((reduce_vec_kernel<ACC, FP16, NSRC>), dim3((unsigned)blocks), dim3(kVecBlock), 0, s, dst + at * 4, t.p[0], cnt, scale,
                           t.p[1], t.p[2], t.p[3], (int)phase);
        at += cnt;
    }
}

template <bool ACC, bool FP16>
void launch_scalar(float* dst, const uint16_t* src, int64_t first, int64_t n, float scale, hipStream_t s) {
    while (first < n) {
        int64_t blocks = (n - first + 255) / 256;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t stop = first + blocks * 256 < n ? first + blocks * 256 : n;
        hipLaunchKernelGGL((reduce_scalar_kernel<ACC, FP16>), dim3((unsigned)blocks), dim3(256), 0, s, dst, src, first, stop, scale);
        first = stop;
    }
}

template <bool ACC, bool FP16>
void launch_reduce(float* dst, const uint16_t* src, int64_t n, float scale, hipStream_t s) {
    int64_t done = 0;
    if (aligned(dst, 16) && aligned(src, 8) && n >= 4) {
        launch_vec<ACC, FP16, 1>(dst, SrcTable{{src}}, n / 4, scale, s);
        done = n / 4 * 4;
    }
    launch_scalar<ACC, FP16>(dst, src, done, n, scale, s);
}

// n_src >= 1 sources into dst, in order, at most kMaxSources per pass; the first pass overwrites unless `acc`.
template <bool FP16>
void launch_sources(float* dst, const uint16_t* const* src, int n_src, int64_t n, float scale, bool acc, hipStream_t s) {
    bool vec = aligned(dst, 16) && n >= 4;
    for (int k = 0; k < n_src; ++k) vec = vec && aligned(src[k], 8);
    if (!vec) {  // a slice at an odd offset: one source per pass through the single-source path
        for (int k = 0; k < n_src; ++k) {
            if (acc || k > 0) launch_reduce<true, FP16>(dst, src[k], n, scale, s);
            else launch_reduce<false, FP16>(dst, src[k], n, scale, s);
        }
        return;
    }
    const int64_t n4 = n / 4;
    for (int k0 = 0; k0 < n_src; k0 += kMaxSources) {
        const int cnt = n_src - k0 < kMaxSources ? n_src - k0 : kMaxSources;
        SrcTable t;
        for (int k = 0; k < kMaxSources; ++k) t.p[k] = k < cnt ? src[k0 + k] : nullptr;
        const bool a = acc || k0 > 0;
#define ELIXIR_SRC_CASE(N)                                            \
    case N:                                                           \
        if (a) launch_vec<true, FP16, N>(dst, t, n4, scale, s);       \
        else launch_vec<false, FP16, N>(dst, t, n4, scale, s);        \
        break;
        switch (cnt) {
            ELIXIR_SRC_CASE(1)
            ELIXIR_SRC_CASE(2)
            ELIXIR_SRC_CASE(3)
            ELIXIR_SRC_CASE(4)
        }
#undef ELIXIR_SRC_CASE
    }
    for (int k = 0; k < n_src && n4 * 4 < n; ++k) {  // the at most 3 elements after the last complete group, source by source
        if (acc || k > 0) launch_scalar<true, FP16>(dst, src[k], n4 * 4, n, scale, s);
        else launch_scalar<false, FP16>(dst, src[k], n4 * 4, n, scale, s);
    }
}

}  // namespace

extern "C" int elixir_grad_reduce_into_chunk_lp(float* d_grad_chunk, int64_t offset, const uint16_t* d_grad_lowp, int lowp_format,
                                                int64_t n, float scale, int accumulate, elixir_stream_t stream) {
    static const char* what = "elixir_grad_reduce_into_chunk";
    if (n < 0 || offset < 0)
        return fail(ELIXIR_EINVAL, "%s: n=%lld, offset=%lld must not be negative", what, (long long)n, (long long)offset);
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (n == 0) return ELIXIR_OK;
    if (!d_grad_chunk || !d_grad_lowp) return fail(ELIXIR_EINVAL, "%s: NULL pointer", what);
    if (!aligned(d_grad_chunk, 4) || !aligned(d_grad_lowp, 2))
        return fail(ELIXIR_EALIGN, "%s: a pointer is not aligned for its element type", what);
    hipStream_t s = (hipStream_t)stream;
    float* dst = d_grad_chunk + offset;
    const bool f16 = lowp_format == ELIXIR_LOWP_FP16;
    if (accumulate) {
        if (f16) launch_reduce<true, true>(dst, d_grad_lowp, n, scale, s);
        else launch_reduce<true, false>(dst, d_grad_lowp, n, scale, s);
    } else {
        if (f16) launch_reduce<false, true>(dst, d_grad_lowp, n, scale, s);
        else launch_reduce<false, false>(dst, d_grad_lowp, n, scale, s);
    }
    ELIXIR_LAUNCH_CHECK("reduce kernel");
    return ELIXIR_OK;
}

extern "C" int elixir_grad_reduce_into_chunk(float* d_grad_chunk, int64_t offset, const uint16_t* d_grad_bf16, int64_t n,
                                             float scale, int accumulate, elixir_stream_t stream) {
    return elixir_grad_reduce_into_chunk_lp(d_grad_chunk, offset, d_grad_bf16, ELIXIR_LOWP_BF16, n, scale, accumulate, stream);
}

extern "C" int elixir_grad_reduce_sources_lp(float* d_grad_chunk, int64_t offset, const uint16_t* const* d_grad_lowp, int n_sources,
                                             int lowp_format, int64_t n, float scale, int accumulate, elixir_stream_t stream) {
    static const char* what = "elixir_grad_reduce_sources";
    if (n < 0 || offset < 0 || n_sources < 0)
        return fail(ELIXIR_EINVAL, "%s: n=%lld, offset=%lld, n_sources=%d must not be negative", what, (long long)n, (long long)offset, n_sources);
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (n == 0 || n_sources == 0) return ELIXIR_OK;
    if (!d_grad_chunk || !d_grad_lowp) return fail(ELIXIR_EINVAL, "%s: NULL pointer", what);
    if (!aligned(d_grad_chunk, 4)) return fail(ELIXIR_EALIGN, "%s: d_grad_chunk is not 4-byte aligned", what);
    for (int k = 0; k < n_sources; ++k) {
        if (!d_grad_lowp[k]) return fail(ELIXIR_EINVAL, "%s: source %d is NULL", what, k);
        if (!aligned(d_grad_lowp[k], 2)) return fail(ELIXIR_EALIGN, "%s: source %d is not 2-byte aligned", what, k);
    }
    hipStream_t s = (hipStream_t)stream;
    if (lowp_format == ELIXIR_LOWP_FP16) launch_sources<true>(d_grad_chunk + offset, d_grad_lowp, n_sources, n, scale, accumulate != 0, s);
    else launch_sources<false>(d_grad_chunk + offset, d_grad_lowp, n_sources, n, scale, accumulate != 0, s);
    ELIXIR_LAUNCH_CHECK("reduce kernel");
    return ELIXIR_OK;
}

namespace {

// Rows of the batched reduction: a tile is what one workgroup handles (kMultiBlock groups of 4 elements).
template <bool ACC, bool FP16>
struct ReduceLaunch {
    float scale;
    hipStream_t s;
    int operator()(const CompactRows& tab, int rows, int64_t longest) const {
        hipLaunchKernelGGL((reduce_rows_kernel<ACC, FP16>), dim3((unsigned)longest, (unsigned)rows), dim3(kMultiBlock), 0, s, tab, scale);
        ELIXIR_LAUNCH_CHECK("reduce_rows_kernel");
        return ELIXIR_OK;
    }
};

template <bool ACC, bool FP16>
struct ReduceRows {
    float* const* d_dst;
    const uint16_t* const* d_src;
    const int64_t* n;
    CompactRowBuilder<16, 8, kMultiBlock, ReduceLaunch<ACC, FP16>> table;
    int rc = ELIXIR_OK;

    void add(int k, int64_t first_tile, int64_t n_tiles) {
        int64_t g0, g1;  // the groups of tensor k that these workgroups handle
        row_piece<16, kMultiBlock>(d_dst[k], n[k] / 4, first_tile, n_tiles, &g0, &g1);
        if (rc == ELIXIR_OK)
            rc = table.add(reinterpret_cast<char*>(d_dst[k] + g0 * 4), reinterpret_cast<const char*>(d_src[k] + g0 * 4), g1 - g0);
    }
    int flush(int64_t) { return rc != ELIXIR_OK ? rc : table.flush(); }
};

template <bool ACC, bool FP16>
int reduce_multi(int T, float* const* d_dst, const uint16_t* const* d_src, const int64_t* n, float scale, hipStream_t s) {
    // tensors that qualify for the vector kernel go through the row plan; a slice at an odd offset or a handful of
    // elements takes the single path, and so do the at most 3 elements after a tensor's last complete group
    auto vec = [&](int k) { return n[k] >= 4 && aligned(d_dst[k], 16) && aligned(d_src[k], 8); };
    for (int k = 0; k < T; ++k) {
        if (n[k] == 0) continue;
        if (!vec(k)) {
            launch_reduce<ACC, FP16>(d_dst[k], d_src[k], n[k], scale, s);
            ELIXIR_LAUNCH_CHECK("reduce kernel");
        } else if (n[k] % 4) {
            hipLaunchKernelGGL((reduce_scalar_kernel<ACC, FP16>), dim3(1), dim3(256), 0, s, d_dst[k], d_src[k], n[k] / 4 * 4, n[k], scale);
            ELIXIR_LAUNCH_CHECK("reduce_scalar_kernel");
        }
    }
    ReduceRows<ACC, FP16> rows{d_dst, d_src, n, CompactRowBuilder<16, 8, kMultiBlock, ReduceLaunch<ACC, FP16>>(ReduceLaunch<ACC, FP16>{scale, s})};
    auto tiles = [&](int k) -> int64_t { return vec(k) ? row_tiles<16, kMultiBlock>(d_dst[k], n[k] / 4) : 0; };
    return plan_rows(T, tiles, 1, kCompactRows, kMaxRowTiles, rows);
}

int elixir_grad_reduce_multi_lp_impl(int n_tensors, float* const* d_dst, const uint16_t* const* d_grad_lowp,
                                     const int64_t* n, int lowp_format, float scale, int accumulate,
                                     elixir_stream_t stream) {
    static const char* what = "elixir_grad_reduce_multi";
    if (n_tensors < 0) return fail(ELIXIR_EINVAL, "%s: n_tensors is negative", what);
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (n_tensors == 0) return ELIXIR_OK;
    if (!d_dst || !d_grad_lowp || !n) return fail(ELIXIR_EINVAL, "%s: NULL table", what);
    for (int k = 0; k < n_tensors; ++k) {
        if (n[k] < 0) return fail(ELIXIR_EINVAL, "%s: n[%d] is negative", what, k);
        if (n[k] == 0) continue;
        if (!d_dst[k] || !d_grad_lowp[k]) return fail(ELIXIR_EINVAL, "%s: NULL pointer for tensor %d", what, k);
        if (!aligned(d_dst[k], 4) || !aligned(d_grad_lowp[k], 2))
            return fail(ELIXIR_EALIGN, "%s: a pointer of tensor %d is not aligned for its element type", what, k);
    }
    hipStream_t s = (hipStream_t)stream;
    const bool f16 = lowp_format == ELIXIR_LOWP_FP16;
    if (accumulate) return f16 ? reduce_multi<true, true>(n_tensors, d_dst, d_grad_lowp, n, scale, s)
                               : reduce_multi<true, false>(n_tensors, d_dst, d_grad_lowp, n, scale, s);
    return f16 ? reduce_multi<false, true>(n_tensors, d_dst, d_grad_lowp, n, scale, s)
               : reduce_multi<false, false>(n_tensors, d_dst, d_grad_lowp, n, scale, s);
}
}  // namespace

extern "C" int elixir_grad_reduce_multi_lp(int n_tensors, float* const* d_dst, const uint16_t* const* d_grad_lowp,
                                           const int64_t* n, int lowp_format, float scale, int accumulate,
                                           elixir_stream_t stream) {
    return no_throw("elixir_grad_reduce_multi_lp", [&] {
        return elixir_grad_reduce_multi_lp_impl(n_tensors, d_dst, d_grad_lowp, n, lowp_format, scale, accumulate,
                                                stream);
    });
}
