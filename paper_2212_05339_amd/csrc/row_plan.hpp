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

}  // namespace elixir
