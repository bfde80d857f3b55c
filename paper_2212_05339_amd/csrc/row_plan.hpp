// Grid rows for the batched kernels (many tensors / many chunks in one launch).  Host only, no allocation.
//
// A batched kernel runs on a grid (row length, rows): row r is a piece of one item (a tensor of the gradient
// reduction, a chunk of the AdamW update), workgroup x of row r works on tile x of that piece, and workgroups past the
// end of a shorter row exit at once.  Workgroups are dispatched x-first, so each row is swept front to back like a
// launch of its own, without the drain and refill between launches.  Measured on MI355X: a workgroup that only finds
// out that it has nothing to do costs about an eighth of a working one, and a further launch about as much as 20K such
// idle workgroups.  The table of rows travels as a kernel argument, which bounds the rows of one launch.
//
// plan_rows cuts every item into pieces of P tiles (P a multiple of `granule`) plus one shorter tail, and hands the rows
// to the caller table by table:
//   * all full pieces first (no idle workgroups, row length P);
//   * then the tails, longest first, a table taking a further tail only while the idle workgroups stay below 1/64 of
//     the working ones + 16K (so tails of similar length share a launch and tiny items get launches of their own);
//   * P is chosen among a handful of candidates (the lengths that occur, and the longest divided by small numbers) as
//     the one with the smallest estimated cost  idle workgroups + 20K * launches;  with lengths that are multiples of
//     each other (the weight matrices of a transformer) this finds the common piece and the grid has no idle tail.
// Tails are ordered with a counting sort over 256 length classes, so the whole plan is O(items) per candidate.
#pragma once
#include <stdint.h>

namespace elixir {

constexpr int kRowWindow = 4096;         // items planned together (index table on the stack); longer lists go window by window
constexpr int64_t kLaunchCost = 20000;   // idle workgroups that cost as much as one more launch
constexpr int kTailClasses = 256;

struct RowTableState {
    int rows = 0;
    int64_t longest = 0, used = 0;
};

// true if a table holding `t` should be launched before a row of `len` tiles is added
inline bool row_is_wasteful(const RowTableState& t, int64_t len) {
    if (t.rows == 0) return false;
    const int64_t longest = len > t.longest ? len : t.longest;
    const int64_t used = t.used + len;
    return longest * (t.rows + 1) - used > used / 64 + 16384;
}

// Estimated cost (idle workgroups + kLaunchCost per launch) of cutting the window's items into pieces of P tiles.
template <class TilesFn>
int64_t row_plan_cost(int i0, int i1, TilesFn& tiles, int64_t P, int max_rows) {
    int64_t full = 0;
    int64_t cnt[kTailClasses] = {}, sum[kTailClasses] = {};
    for (int i = i0; i < i1; ++i) {
        const int64_t t = tiles(i);
        if (t <= 0) continue;
        full += t / P;
        const int64_t tail = t % P;
        if (tail) {
            const int b = (int)(tail * kTailClasses / P);
            ++cnt[b];
            sum[b] += tail;
        }
    }
    int64_t launches = full / max_rows, idle = 0;
    RowTableState tab;
    tab.rows = (int)(full % max_rows);
    tab.longest = tab.rows ? P : 0;
    tab.used = (int64_t)tab.rows * P;
    for (int b = kTailClasses - 1; b >= 0; --b) {
        if (!cnt[b]) continue;
        const int64_t len = sum[b] / cnt[b];  // the class's mean stands for its members
        for (int64_t k = 0; k < cnt[b]; ++k) {
            if (tab.rows == max_rows || row_is_wasteful(tab, len)) {
                idle += tab.longest * tab.rows - tab.used;
                ++launches;
                tab = RowTableState();
            }
            ++tab.rows;
            tab.used += len;
            if (len > tab.longest) tab.longest = len;
        }
    }
    if (tab.rows) {
        idle += tab.longest * tab.rows - tab.used;
        ++launches;
    }
    return idle + kLaunchCost * launches;
}

// Sink: void add(int item, int64_t first_tile, int64_t n_tiles);  int flush(int64_t row_length) -- launches the rows
// added since the last flush on a grid whose rows are row_length tiles long; returns a status (0 = OK).
// tiles(i): tiles of item i, 0 to leave the item out.  max_piece: upper bound on a row's length (the grid's x limit).
template <class TilesFn, class Sink>
int plan_rows(int n_items, TilesFn tiles, int64_t granule, int max_rows, int64_t max_piece, Sink& sink) {
    for (int i0 = 0; i0 < n_items; i0 += kRowWindow) {
        const int i1 = n_items - i0 < kRowWindow ? n_items : i0 + kRowWindow;
        int64_t longest = 0;
        for (int i = i0; i < i1; ++i)
            if (tiles(i) > longest) longest = tiles(i);
        if (longest == 0) continue;
        // ---- candidates for the piece length
        int64_t cand[24];
        int n_cand = 0;
        auto offer = [&](int64_t p) {
            p = (p + granule - 1) / granule * granule;
            if (p > max_piece) p = max_piece / granule * granule;
            if (p < granule) p = granule;
            for (int k = 0; k < n_cand; ++k)
                if (cand[k] == p) return;
            if (n_cand < 24) cand[n_cand++] = p;
        };
        offer(longest);
        static const int kDiv[] = {2, 3, 4, 6, 8, 12, 16, 24, 32};
        for (int d : kDiv) offer(longest / d);
        for (int i = i0; i < i1 && n_cand < 20; ++i)  // lengths that occur, as far as they are not dwarfed by the longest
            if (tiles(i) * 64 >= longest) offer(tiles(i));
        int64_t P = cand[0], best = -1;
        for (int k = 0; k < n_cand; ++k) {
            const int64_t c = row_plan_cost(i0, i1, tiles, cand[k], max_rows);
            if (best < 0 || c < best || (c == best && cand[k] > P)) {
                best = c;
                P = cand[k];
            }
        }
        // ---- full pieces
        RowTableState tab;
        auto flush = [&]() -> int {
            if (tab.rows == 0) return 0;
            const int rc = sink.flush(tab.longest);
            tab = RowTableState();
            return rc;
        };
        for (int i = i0; i < i1; ++i) {
            const int64_t t = tiles(i);
            for (int64_t f = 0; f + P <= t; f += P) {
                if (tab.rows == max_rows)
                    if (const int rc = flush()) return rc;
                sink.add(i, f, P);
                ++tab.rows;
                tab.used += P;
                tab.longest = P;
            }
        }
        // ---- tails, longest class first (counting sort of the window's items by tail class)
        int start[kTailClasses + 1] = {};
        for (int i = i0; i < i1; ++i) {
            const int64_t t = tiles(i);
            if (t > 0 && t % P) ++start[(int)((t % P) * kTailClasses / P)];
        }
        int at = 0;
        for (int b = kTailClasses - 1; b >= 0; --b) {  // start[b] = position of class b's first item, classes descending
            const int c = start[b];
            start[b] = at;
            at += c;
        }
        int order[kRowWindow];
        for (int i = i0; i < i1; ++i) {
            const int64_t t = tiles(i);
            if (t > 0 && t % P) order[start[(int)((t % P) * kTailClasses / P)]++] = i;
        }
        for (int k = 0; k < at; ++k) {
            const int i = order[k];
            const int64_t t = tiles(i), tail = t % P;
            if (tab.rows == max_rows || row_is_wasteful(tab, tail))
                if (const int rc = flush()) return rc;
            sink.add(i, t - tail, tail);
            ++tab.rows;
            tab.used += tail;
            if (tail > tab.longest) tab.longest = tail;
        }
        if (const int rc = flush()) return rc;
    }
    return 0;
}

// ---- the table of rows as it travels in the kernel arguments ----------------------------------------------------------
//
// Every launch boundary costs (the chip drains and refills), so a launch should carry as many rows as the 4 KB of kernel
// arguments allow.  Rows are therefore stored compactly: two base addresses per launch (the lowest destination and the
// lowest source among its rows) and per row two 32-bit offsets from them, in units of UNIT bytes, and a 32-bit count:
// 12 bytes instead of 24, 336 rows instead of 160.  A row whose offset would not fit (addresses more than 2^32 units
// apart within one launch) makes the builder launch what it has and start a new table, so any set of rows is accepted.
// A row may have no source (a fill): its source offset is kNoSource.
//
// Where a row starts matters as well: a wavefront moves TILE consecutive units, and when that KiB of the destination
// straddles a KiB boundary every boundary line is written by two wavefronts (measured on the gradient reduction, rows of
// 2.56M elements: 82.9% of the HBM peak with aligned rows, 79.3% with every row 512 bytes past a boundary).  So the
// destination base is a multiple of TILE units, the kernels take  phase = dst_off mod TILE  of a row as the number of
// lanes that its first workgroup leaves idle, and every later workgroup of the row is aligned: workgroup x handles
// units [x TILE - phase, (x + 1) TILE - phase) of the row.  row_phase / row_tiles / row_piece below are the host side
// of that rule.
constexpr int kCompactRows = 336;
constexpr uint32_t kNoSource = 0xFFFFFFFFu;
struct CompactRows {
    char* dst_base;
    const char* src_base;
    uint32_t dst_off[kCompactRows];   // units of DST_UNIT bytes from dst_base
    uint32_t src_off[kCompactRows];   // units of SRC_UNIT bytes from src_base, or kNoSource
    uint32_t count[kCompactRows];     // what the kernel counts (groups of 4 elements, 16-byte units)
};
static_assert(sizeof(CompactRows) + 16 <= 4096, "the table (and a scalar beside it) must fit the kernel arguments");

// Collects rows and hands complete tables to launch(table, rows, longest row in tiles).  DST_UNIT / SRC_UNIT: bytes per
// offset unit (the addresses are multiples of them); TILE: count units per workgroup.
template <int DST_UNIT, int SRC_UNIT, int TILE, class Launch>
struct CompactRowBuilder {
    Launch launch;
    char* dst[kCompactRows];
    const char* src[kCompactRows];
    CompactRows tab;
    int rows = 0;
    int64_t longest = 0;   // tiles
    uintptr_t d_lo = 0, d_hi = 0, s_lo = 0, s_hi = 0;
    bool any_src = false;

    explicit CompactRowBuilder(Launch l) : launch(l) {}

    static constexpr uint64_t kSpan = 0xFFFFFFFEull;  // largest offset, in units (kNoSource stays free)

    static constexpr uintptr_t kBaseGrain = (uintptr_t)DST_UNIT * TILE;  // the destination base is a multiple of this

    int add(char* d, const char* s, int64_t count) {
        const uintptr_t da = reinterpret_cast<uintptr_t>(d), sa = reinterpret_cast<uintptr_t>(s);
        if (rows) {
            const uintptr_t nd_lo = (da < d_lo ? da : d_lo) / kBaseGrain * kBaseGrain, nd_hi = da > d_hi ? da : d_hi;
            uintptr_t ns_lo = s_lo, ns_hi = s_hi;
            if (s && any_src) {
                ns_lo = sa < s_lo ? sa : s_lo;
                ns_hi = sa > s_hi ? sa : s_hi;
            } else if (s) {
                ns_lo = ns_hi = sa;
            }
            const bool fits = (nd_hi - nd_lo) / DST_UNIT <= kSpan && (!(s || any_src) || (ns_hi - ns_lo) / SRC_UNIT <= kSpan);
            if (!fits || rows == kCompactRows)
                if (const int rc = flush()) return rc;
        }
        if (!rows) {
            d_lo = d_hi = da;
            any_src = false;
        }
        if (da < d_lo) d_lo = da;
        if (da > d_hi) d_hi = da;
        if (s) {
            if (!any_src) s_lo = s_hi = sa;
            if (sa < s_lo) s_lo = sa;
            if (sa > s_hi) s_hi = sa;
            any_src = true;
        }
        dst[rows] = d;
        src[rows] = s;
        tab.count[rows] = (uint32_t)count;
        const int64_t t = (count + (int64_t)(da / DST_UNIT % TILE) + TILE - 1) / TILE;  // the first workgroup starts `phase` lanes in
        if (t > longest) longest = t;
        ++rows;
        return 0;
    }
    int flush() {
        if (!rows) return 0;
        const uintptr_t d_base = d_lo / kBaseGrain * kBaseGrain;
        tab.dst_base = reinterpret_cast<char*>(d_base);
        tab.src_base = any_src ? reinterpret_cast<const char*>(s_lo) : nullptr;
        for (int r = 0; r < rows; ++r) {
            tab.dst_off[r] = (uint32_t)((reinterpret_cast<uintptr_t>(dst[r]) - d_base) / DST_UNIT);
            tab.src_off[r] = src[r] ? (uint32_t)((reinterpret_cast<uintptr_t>(src[r]) - s_lo) / SRC_UNIT) : kNoSource;
        }
        for (int r = rows; r < kCompactRows; ++r) {
            tab.dst_off[r] = 0;
            tab.src_off[r] = kNoSource;
            tab.count[r] = 0;
        }
        const int rc = launch(tab, rows, longest);
        rows = 0;
        longest = 0;
        return rc;
    }
};

// Host side of the alignment rule for an item of n units whose destination starts at address d.
template <int DST_UNIT, int TILE>
inline int64_t row_phase(const void* d) {
    return (int64_t)(reinterpret_cast<uintptr_t>(d) / DST_UNIT % TILE);
}
template <int DST_UNIT, int TILE>
inline int64_t row_tiles(const void* d, int64_t n) {  // workgroups the item takes
    return (n + row_phase<DST_UNIT, TILE>(d) + TILE - 1) / TILE;
}
// The units [*begin, *end) of the item that its workgroups [first_tile, first_tile + n_tiles) handle.
template <int DST_UNIT, int TILE>
inline void row_piece(const void* d, int64_t n, int64_t first_tile, int64_t n_tiles, int64_t* begin, int64_t* end) {
    const int64_t phase = row_phase<DST_UNIT, TILE>(d);
    *begin = first_tile ? first_tile * TILE - phase : 0;
    *end = (first_tile + n_tiles) * TILE - phase;
    if (*end > n) *end = n;
}

}  // namespace elixir
