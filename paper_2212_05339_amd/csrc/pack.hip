// elixir_chunk_pack / elixir_chunk_unpack: bit copies between parameter tensors and one chunk.
//
// A chunk is the concatenation of a group of flattened parameters (paper Sec. 3
// "Chunk", Fig. 3 left).  The host turns the request into a list of byte
// segments (source, destination, length; for pack also the gaps, which are
// zero-filled).  Two kernels move them, both with the table as a kernel
// argument, so no device memory is allocated or copied for it:
//   * the tile kernel cuts the segments into tiles of kTileBytes, one
//     single-wavefront workgroup per tile, which finds its segment by a search
//     over the table and moves the tile with the widest access both addresses
//     allow (16, 4 or 2 bytes per lane): any alignment, 96 segments a launch;
//   * the row kernel takes segments whose two addresses are 16-byte aligned as
//     the rows of a 2-D grid (row_plan.hpp): no search, 336 rows a launch, rows
//     started on KiB boundaries of the destination.
// Workgroups are dispatched in index order, so source and destination are swept
// as sequential fronts (one slice: 6.8 TB/s; 6.6 TB/s with 256-thread workgroups
// and 4 KiB tiles; ~5.4 TB/s for hipMemcpy D2D).
// Traffic: read + write of every byte (write only for gaps).
#include <stdlib.h>

#include <algorithm>

#include "common.hpp"
#include "row_plan.hpp"

using namespace elixir;

namespace {

constexpr int kMaxSeg = 96;
constexpr int kCopyBlock = 64;                     // one wavefront per workgroup
constexpr int64_t kTileBytes = kCopyBlock * 16;   // one 128-bit access per lane, one workgroup per tile
constexpr uint64_t kMaxTilesPerLaunch = ((1ull << 32) - 1) / kCopyBlock;  // HIP refuses grids of 2^32 threads or more in x (64 GiB per launch)

struct SegTable {
    const char* src[kMaxSeg];  // nullptr: fill with zero bits
    char* dst[kMaxSeg];
    int64_t bytes[kMaxSeg];
    uint32_t tile_begin[kMaxSeg + 1];
    int n_seg;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename W>
__device__ __forceinline__ void move_units(char* dst, const char* src, int64_t n_units) {
    W* D = reinterpret_cast<W*>(dst);
    const W* S = reinterpret_cast<const W*>(src);
    if (src) {
        for (int64_t i = threadIdx.x; i < n_units; i += kCopyBlock) __builtin_nontemporal_store(__builtin_nontemporal_load(S + i), D + i);
    } else {
        const W z = W(0);
        for (int64_t i = threadIdx.x; i < n_units; i += kCopyBlock) __builtin_nontemporal_store(z, D + i);
    }
}

__global__ __launch_bounds__(kCopyBlock) void segment_copy_kernel(SegTable tab) {
    // which segment owns this tile: last s with tile_begin[s] <= blockIdx.x
    int lo = 0, hi = tab.n_seg;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab.tile_begin[mid] <= blockIdx.x) lo = mid;
        else hi = mid;
    }
    const int64_t off = (int64_t)(blockIdx.x - tab.tile_begin[lo]) * kTileBytes;
    int64_t len = tab.bytes[lo] - off;
    if (len > kTileBytes) len = kTileBytes;
    const char* src = tab.src[lo] ? tab.src[lo] + off : nullptr;
    char* dst = tab.dst[lo] + off;
    const uintptr_t a = reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src);
    int64_t done;
    if ((a & 15) == 0) {
        move_units<u32x4>(dst, src, len >> 4);
        done = len & ~(int64_t)15;
    } else if ((a & 3) == 0) {
        move_units<uint32_t>(dst, src, len >> 2);
        done = len & ~(int64_t)3;
    } else {
        done = 0;
    }
    if (done < len) move_units<uint16_t>(dst + done, src ? src + done : nullptr, (len - done) >> 1);
}

// Slices as the rows of a 2-D grid (see row_plan.hpp): row r moves count[r] units of 16 bytes from its source (none:
// zero bits) to its destination, both 16-byte aligned, one unit per lane, workgroup x of the row its x-th KiB.  No
// search for the owner of a tile, up to 336 rows per launch.
constexpr int64_t kMaxRowTiles = 1ll << 22;

__global__ __launch_bounds__(kCopyBlock) void copy_rows_kernel(CompactRows tab) {
    const int r = blockIdx.y;
    const uint32_t d_off = tab.dst_off[r], s_off = tab.src_off[r], n16 = tab.count[r];
    char* dst_base = tab.dst_base;
    const char* src_base = tab.src_base;
    asm volatile("" ::"s"(d_off), "s"(s_off), "s"(n16), "s"(dst_base), "s"(src_base));  // one round of scalar loads
    const uint32_t phase = d_off % kCopyBlock;  // dst_base is KiB-aligned: the row starts this many units past a KiB boundary
    if (blockIdx.x * kCopyBlock >= n16 + phase) return;  // past the end of a shorter row (uniform per workgroup)
    const int32_t i = (int32_t)(blockIdx.x * kCopyBlock + threadIdx.x) - (int32_t)phase;  // the first workgroup's first lanes idle
    if (i >= 0 && (uint32_t)i < n16) {
        u32x4 v = u32x4(0);
        if (s_off != kNoSource) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src_base) + s_off + i);
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst_base) + d_off + i);
    }
}

struct Seg {
    const char* src;
    char* dst;
    int64_t bytes;
};

// The slice tables of a call: on the stack for up to N entries (a chunk holds a few dozen tensors), on the heap only
// beyond that, so that the usual call allocates nothing.
template <typename T, int N>
struct Table {
    T local[N];
    T* p = local;
    size_t n = 0, cap = N;
    Table() = default;
    Table(const Table&) = delete;
    Table& operator=(const Table&) = delete;
    ~Table() {
        if (p != local) free(p);
    }
    bool reserve(size_t want) {
        if (want <= cap) return true;
        T* q = static_cast<T*>(malloc(want * sizeof(T)));
        if (!q) return false;
        for (size_t i = 0; i < n; ++i) q[i] = p[i];
        if (p != local) free(p);
        p = q;
        cap = want;
        return true;
    }
    void push(const T& v) { p[n++] = v; }  // the caller has reserved
};
constexpr int kStackSlices = 512;
typedef Table<int, kStackSlices> OrderTable;
typedef Table<Seg, 2 * kStackSlices + 1> SegTableHost;

// Segments [i, end) of the table, 96 to a launch.
int launch_segments(const SegTableHost& segs, hipStream_t s, const char* what, size_t i = 0, size_t end = (size_t)-1) {
    if (end > segs.n) end = segs.n;
    while (i < end) {
        SegTable tab;
        tab.n_seg = 0;
        uint64_t tiles = 0;
        while (i < end && tab.n_seg < kMaxSeg) {
            const Seg& g = segs.p[i];
            const uint64_t t = (uint64_t)((g.bytes + kTileBytes - 1) / kTileBytes);
            if (tiles + t > kMaxTilesPerLaunch) break;  // the rest goes to the next launch
            tab.src[tab.n_seg] = g.src;
            tab.dst[tab.n_seg] = g.dst;
            tab.bytes[tab.n_seg] = g.bytes;
            tab.tile_begin[tab.n_seg] = (uint32_t)tiles;
            tiles += t;
            ++tab.n_seg;
            ++i;
        }
        if (tab.n_seg == 0) return fail(ELIXIR_EINVAL, "%s: a single slice is too large for one launch", what);
        for (int j = tab.n_seg; j <= kMaxSeg; ++j) tab.tile_begin[j] = (uint32_t)tiles;
        for (int j = tab.n_seg; j < kMaxSeg; ++j) { tab.src[j] = nullptr; tab.dst[j] = nullptr; tab.bytes[j] = 0; }
        hipLaunchKernelGGL(segment_copy_kernel, dim3((unsigned)tiles), dim3(kCopyBlock), 0, s, tab);
        ELIXIR_LAUNCH_CHECK(what);
    }
    return ELIXIR_OK;
}

// All segments of the table in few launches: those whose two addresses are 16-byte aligned go through the row plan
// (whole 16-byte units), the others and the last bytes of a segment through the tile kernel above.
struct CopyLaunch {
    hipStream_t s;
    const char* what;
    int operator()(const CompactRows& tab, int rows, int64_t longest) const {
        hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)longest, (unsigned)rows), dim3(kCopyBlock), 0, s, tab);
        ELIXIR_LAUNCH_CHECK(what);
        return ELIXIR_OK;
    }
};

struct CopyRows {
    const SegTableHost& segs;
    CompactRowBuilder<16, 16, kCopyBlock, CopyLaunch> table;
    int rc = ELIXIR_OK;

    void add(int k, int64_t first_tile, int64_t n_tiles) {
        const Seg& g = segs.p[k];
        int64_t u0, u1;  // the 16-byte units of the segment that these workgroups move
        row_piece<16, kCopyBlock>(g.dst, g.bytes / 16, first_tile, n_tiles, &u0, &u1);
        if (rc == ELIXIR_OK) rc = table.add(g.dst + u0 * 16, g.src ? g.src + u0 * 16 : nullptr, u1 - u0);
    }
    int flush(int64_t) { return rc != ELIXIR_OK ? rc : table.flush(); }
};

int launch_rows(const SegTableHost& segs, hipStream_t s, const char* what) {
    if (segs.n > (size_t)INT32_MAX) return fail(ELIXIR_ECAP, "%s: too many slices", what);
    auto vec = [&](int k) {
        const Seg& g = segs.p[k];
        return g.bytes >= 16 && aligned(g.dst, 16) && aligned(g.src, 16);  // a null source (zero fill) counts as aligned
    };
    // what the rows do not take: unaligned segments whole, and the last bytes (fewer than 16) of the others
    SegTableHost rest;
    size_t n_rest = 0;
    for (size_t k = 0; k < segs.n; ++k) n_rest += !vec((int)k) || segs.p[k].bytes % 16;
    if (!rest.reserve(n_rest)) return fail(ELIXIR_EINVAL, "%s: out of host memory", what);
    for (size_t k = 0; k < segs.n; ++k) {
        const Seg& g = segs.p[k];
        if (g.bytes == 0) continue;
        if (!vec((int)k)) rest.push(g);
        else if (g.bytes % 16) {
            const int64_t done = g.bytes / 16 * 16;
            rest.push({g.src ? g.src + done : nullptr, g.dst + done, g.bytes - done});
        }
    }
    if (rest.n)
        if (const int rc = launch_segments(rest, s, what)) return rc;
    CopyRows rows{segs, CompactRowBuilder<16, 16, kCopyBlock, CopyLaunch>(CopyLaunch{s, what})};
    auto tiles = [&](int k) -> int64_t { return vec(k) ? row_tiles<16, kCopyBlock>(segs.p[k].dst, segs.p[k].bytes / 16) : 0; };
    return plan_rows((int)segs.n, tiles, 1, kCompactRows, kMaxRowTiles, rows);
}

// The segments of ONE chunk.  A call is at least one launch either way; measured on the chunks of the 1.5B set: with
// one slice per chunk the rows move 81% of the HBM peak (the tile kernel 78%), with the chunk's two dozen tensors the
// tile kernel's single launch moves 77% where the rows need a second launch for the small tensors and reach 75%.
constexpr size_t kFewSegments = 4;
int launch_chunk(const SegTableHost& segs, hipStream_t s, const char* what) {
    return segs.n <= kFewSegments ? launch_rows(segs, s, what) : launch_segments(segs, s, what);
}

// Validates the slices and returns their indices ordered by offset (empty slices dropped).
int check_slices(const char* what, const void* chunk, int64_t chunk_elems, int elem_size, const void* const* tensors,
                 const int64_t* numel, const int64_t* offset, int T, OrderTable* order) {
    if (chunk_elems < 0 || T < 0) return fail(ELIXIR_EINVAL, "%s: negative chunk_elems or T", what);
    if (elem_size != 2 && elem_size != 4) return fail(ELIXIR_EINVAL, "%s: elem_size=%d, must be 2 or 4", what, elem_size);
    if ((uint64_t)chunk_elems > kMaxTilesPerLaunch * (uint64_t)kTileBytes / (uint64_t)elem_size)  // no slice or gap can then exceed a launch
        return fail(ELIXIR_ECAP, "%s: a chunk of %lld elements exceeds the %llu bytes one launch moves", what, (long long)chunk_elems,
                    (unsigned long long)(kMaxTilesPerLaunch * (uint64_t)kTileBytes));
    if (chunk_elems > 0 && !chunk) return fail(ELIXIR_EINVAL, "%s: chunk is NULL", what);
    if (T > 0 && (!tensors || !numel || !offset)) return fail(ELIXIR_EINVAL, "%s: NULL table", what);
    if (!aligned(chunk, (size_t)elem_size)) return fail(ELIXIR_EALIGN, "%s: chunk not aligned to elem_size", what);
    order->n = 0;
    if (!order->reserve((size_t)T)) return fail(ELIXIR_EINVAL, "%s: out of host memory for %d slices", what, T);
    for (int i = 0; i < T; ++i) {
        if (numel[i] < 0 || offset[i] < 0 || offset[i] > chunk_elems || numel[i] > chunk_elems - offset[i])
            return fail(ELIXIR_EINVAL, "%s: slice %d (offset %lld, numel %lld) leaves the chunk of %lld elements", what, i,
                        (long long)offset[i], (long long)numel[i], (long long)chunk_elems);
        if (numel[i] == 0) continue;
        if (!tensors[i]) return fail(ELIXIR_EINVAL, "%s: tensors[%d] is NULL", what, i);
        if (!aligned(tensors[i], (size_t)elem_size)) return fail(ELIXIR_EALIGN, "%s: tensors[%d] not aligned to elem_size", what, i);
        order->push(i);
    }
    std::sort(order->p, order->p + order->n, [&](int a, int b) { return offset[a] < offset[b]; });
    for (size_t k = 1; k < order->n; ++k) {
        const int a = order->p[k - 1], b = order->p[k];
        if (offset[a] + numel[a] > offset[b])
            return fail(ELIXIR_EINVAL, "%s: slices %d and %d overlap", what, a, b);
    }
    return ELIXIR_OK;
}

int elixir_chunk_pack_impl(void* d_chunk, int64_t chunk_elems, int elem_size, const void* const* tensors,
                           const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream) {
    static const char* what = "elixir_chunk_pack";
    OrderTable order;
    const int rc = check_slices(what, d_chunk, chunk_elems, elem_size, tensors, numel, offset, T, &order);
    if (rc != ELIXIR_OK) return rc;
    char* base = static_cast<char*>(d_chunk);
    const int64_t es = elem_size;
    SegTableHost segs;
    if (!segs.reserve(2 * order.n + 1)) return fail(ELIXIR_EINVAL, "%s: out of host memory for %d slices", what, T);
    int64_t pos = 0;  // first element not yet covered
    for (size_t k = 0; k < order.n; ++k) {
        const int i = order.p[k];
        if (offset[i] > pos) segs.push({nullptr, base + pos * es, (offset[i] - pos) * es});
        segs.push({static_cast<const char*>(tensors[i]), base + offset[i] * es, numel[i] * es});
        pos = offset[i] + numel[i];
    }
    if (pos < chunk_elems) segs.push({nullptr, base + pos * es, (chunk_elems - pos) * es});
    return launch_chunk(segs, (hipStream_t)stream, what);
}
}  // namespace

extern "C" int elixir_chunk_pack(void* d_chunk, int64_t chunk_elems, int elem_size, const void* const* tensors,
                                 const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream) {
    return no_throw("elixir_chunk_pack", [&] {
        return elixir_chunk_pack_impl(d_chunk, chunk_elems, elem_size, tensors, numel, offset, T, stream);
    });
}

namespace {
int elixir_chunk_unpack_impl(const void* d_chunk, int64_t chunk_elems, int elem_size, void* const* tensors,
                             const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream) {
    static const char* what = "elixir_chunk_unpack";
    OrderTable order;
    const int rc = check_slices(what, d_chunk, chunk_elems, elem_size, tensors, numel, offset, T, &order);
    if (rc != ELIXIR_OK) return rc;
    const char* base = static_cast<const char*>(d_chunk);
    const int64_t es = elem_size;
    SegTableHost segs;
    if (!segs.reserve(order.n)) return fail(ELIXIR_EINVAL, "%s: out of host memory for %d slices", what, T);
    for (size_t k = 0; k < order.n; ++k) {
        const int i = order.p[k];
        segs.push({base + offset[i] * es, static_cast<char*>(tensors[i]), numel[i] * es});
    }
    return launch_chunk(segs, (hipStream_t)stream, what);
}
}  // namespace

extern "C" int elixir_chunk_unpack(const void* d_chunk, int64_t chunk_elems, int elem_size, void* const* tensors,
                                   const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream) {
    return no_throw("elixir_chunk_unpack", [&] {
        return elixir_chunk_unpack_impl(d_chunk, chunk_elems, elem_size, tensors, numel, offset, T, stream);
    });
}

// ---- a whole parameter set at once ------------------------------------------------------------------------------
//
// The per-chunk calls above cost one launch per chunk; at set-up a trainer packs every chunk, and the launch boundaries
// then show (26 launches for the 1.5B set against a handful here).  These take the layout plan as it stands: tensor i occupies
// the linear element range [chunk_id[i] * C + offset[i], + numel[i]) of the chunk sequence, so a tensor longer than the
// rest of its chunk simply continues at the start of the next one.

namespace {

template <bool PACK>
int chunks_copy(const char* what, void* const* d_chunks, int n_chunks, int64_t chunk_elems, int elem_size, const void* const* tensors,
                const int64_t* numel, const int64_t* chunk_id, const int64_t* offset, int T, hipStream_t stream) {
    if (n_chunks < 0 || T < 0 || chunk_elems <= 0) return fail(ELIXIR_EINVAL, "%s: negative n_chunks or T, or chunk_elems not positive", what);
    if (elem_size != 2 && elem_size != 4) return fail(ELIXIR_EINVAL, "%s: elem_size=%d, must be 2 or 4", what, elem_size);
    if ((uint64_t)chunk_elems > kMaxTilesPerLaunch * (uint64_t)kTileBytes / (uint64_t)elem_size)
        return fail(ELIXIR_ECAP, "%s: a chunk of %lld elements exceeds what one launch moves", what, (long long)chunk_elems);
    if ((n_chunks > 0 && !d_chunks) || (T > 0 && (!tensors || !numel || !chunk_id || !offset))) return fail(ELIXIR_EINVAL, "%s: NULL table", what);
    for (int c = 0; c < n_chunks; ++c) {
        if (!d_chunks[c]) return fail(ELIXIR_EINVAL, "%s: d_chunks[%d] is NULL", what, c);
        if (!aligned(d_chunks[c], (size_t)elem_size)) return fail(ELIXIR_EALIGN, "%s: d_chunks[%d] not aligned to elem_size", what, c);
    }
    const int64_t C = chunk_elems, total = C * (int64_t)n_chunks, es = elem_size;
    OrderTable order;
    if (!order.reserve((size_t)T)) return fail(ELIXIR_EINVAL, "%s: out of host memory for %d tensors", what, T);
    auto start = [&](int i) { return chunk_id[i] * C + offset[i]; };
    size_t n_pieces = 0;
    for (int i = 0; i < T; ++i) {
        if (numel[i] < 0 || chunk_id[i] < 0 || offset[i] < 0 || offset[i] >= C || chunk_id[i] >= n_chunks || numel[i] > total - start(i))
            return fail(ELIXIR_EINVAL, "%s: tensor %d (chunk %lld, offset %lld, numel %lld) leaves the %d chunks of %lld elements", what, i,
                        (long long)chunk_id[i], (long long)offset[i], (long long)numel[i], n_chunks, (long long)C);
        if (numel[i] == 0) continue;
        if (!tensors[i]) return fail(ELIXIR_EINVAL, "%s: tensors[%d] is NULL", what, i);
        if (!aligned(tensors[i], (size_t)elem_size)) return fail(ELIXIR_EALIGN, "%s: tensors[%d] not aligned to elem_size", what, i);
        order.push(i);
        n_pieces += (size_t)((offset[i] + numel[i] + C - 1) / C);
    }
    std::sort(order.p, order.p + order.n, [&](int a, int b) { return start(a) < start(b); });
    for (size_t k = 1; k < order.n; ++k)
        if (start(order.p[k - 1]) + numel[order.p[k - 1]] > start(order.p[k]))
            return fail(ELIXIR_EINVAL, "%s: tensors %d and %d overlap", what, order.p[k - 1], order.p[k]);
    SegTableHost segs;
    if (!segs.reserve(2 * n_pieces + 2 * (size_t)n_chunks + 2)) return fail(ELIXIR_EINVAL, "%s: out of host memory", what);
    // All slices are collected first (cut at chunk boundaries), then launched as rows: measured on the 1.5B set, one
    // tile-kernel launch per chunk moves 77% of the HBM peak (26 launches with 5-7 us between them, and a search over
    // the launch's table in every workgroup), tile-kernel launches of 96 slices across chunks 75%.
    // a run of the linear range, cut at chunk boundaries: src == nullptr fills with zero bits (pack only)
    auto emit = [&](int64_t lin, int64_t count, const char* src) {
        while (count > 0) {
            const int64_t c = lin / C, o = lin % C, take = count < C - o ? count : C - o;
            char* chunk = static_cast<char*>(d_chunks[c]) + o * es;
            if (PACK) segs.push({src, chunk, take * es});
            else segs.push({chunk, const_cast<char*>(src), take * es});
            if (src) src += take * es;
            lin += take;
            count -= take;
        }
    };
    int64_t pos = 0;
    for (size_t k = 0; k < order.n; ++k) {
        const int i = order.p[k];
        if (PACK && start(i) > pos) emit(pos, start(i) - pos, nullptr);
        emit(start(i), numel[i], static_cast<const char*>(tensors[i]));
        pos = start(i) + numel[i];
    }
    if (PACK && pos < total) emit(pos, total - pos, nullptr);
    return launch_rows(segs, stream, what);
}

}  // namespace

extern "C" int elixir_chunks_pack(void* const* d_chunks, int n_chunks, int64_t chunk_elems, int elem_size, const void* const* tensors,
                                  const int64_t* numel, const int64_t* chunk_id, const int64_t* offset, int T, elixir_stream_t stream) {
    return no_throw("elixir_chunks_pack", [&] {
        return chunks_copy<true>("elixir_chunks_pack", d_chunks, n_chunks, chunk_elems, elem_size, tensors, numel, chunk_id, offset, T,
                                 (hipStream_t)stream);
    });
}

extern "C" int elixir_chunks_unpack(const void* const* d_chunks, int n_chunks, int64_t chunk_elems, int elem_size, void* const* tensors,
                                    const int64_t* numel, const int64_t* chunk_id, const int64_t* offset, int T, elixir_stream_t stream) {
    return no_throw("elixir_chunks_unpack", [&] {
        return chunks_copy<false>("elixir_chunks_unpack", const_cast<void* const*>(d_chunks), n_chunks, chunk_elems, elem_size,
                                  const_cast<const void* const*>(tensors), numel, chunk_id, offset, T, (hipStream_t)stream);
    });
}
