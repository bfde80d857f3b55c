// Chunk layout planner (host, integers only).
//
// Grouping rule of the paper (App. A.2): parameters are visited in their order
// of use; one chunk is "current"; a parameter is appended to it when it fits,
// otherwise the chunk is closed and a new one is opened.  The paper does not
// say what happens to a parameter longer than a chunk; here it takes fresh
// consecutive chunks and the remainder of its last chunk stays open.
#include <vector>

#include "common.hpp"

using namespace elixir;

namespace {

struct Planner {
    int64_t C, align;
    std::vector<int64_t> used;  // elements in use, per chunk

    int64_t round_up(int64_t x) const { return (x + align - 1) / align * align; }

    // n elements starting at offset 0 of a new chunk, continuing through as many chunks as it takes
    void lay_from_new_chunk(int64_t n) {
        do {
            const int64_t take = n < C ? n : C;
            used.push_back(take);
            n -= take;
        } while (n > 0);
    }

    bool try_append(size_t c, int64_t n, int64_t* off) {
        const int64_t start = round_up(used[c]);
        if (start + n > C) return false;
        *off = start;
        used[c] = start + n;
        return true;
    }

    void place(int64_t n, int policy, int64_t* cid, int64_t* off) {
        if (policy == ELIXIR_LAYOUT_DENSE) {
            if (used.empty()) used.push_back(0);
            size_t c = used.size() - 1;
            int64_t start = round_up(used[c]);
            if (start >= C && n > 0) {
                used.push_back(0);
                ++c;
                start = 0;
            }
            *cid = (int64_t)c;
            *off = start;
            const int64_t room = C - start;
            const int64_t take = n < room ? n : room;
            used[c] = start + take;
            if (n > take) lay_from_new_chunk(n - take);
            return;
        }
        if (n > C) {
            *cid = (int64_t)used.size();
            *off = 0;
            lay_from_new_chunk(n);
            return;
        }
        const size_t first = (policy == ELIXIR_LAYOUT_FIRST_FIT || used.empty()) ? 0 : used.size() - 1;
        for (size_t c = first; c < used.size(); ++c) {
            if (try_append(c, n, off)) {
                *cid = (int64_t)c;
                return;
            }
        }
        *cid = (int64_t)used.size();
        *off = 0;
        used.push_back(n);
    }
};

int elixir_layout_plan_impl(const int64_t* numel, int T, int64_t chunk_elems, int policy, int64_t align_elems,
                            int64_t* chunk_id, int64_t* offset, int64_t* n_chunks, int64_t* valid_len,
                            int64_t valid_cap) {
    if (T < 0 || (T > 0 && (!numel || !chunk_id || !offset)) || !n_chunks)
        return fail(ELIXIR_EINVAL, "elixir_layout_plan: NULL argument or negative T");
    if (chunk_elems <= 0 || align_elems <= 0 || chunk_elems % align_elems != 0)
        return fail(ELIXIR_EINVAL, "elixir_layout_plan: chunk_elems=%lld must be a positive multiple of align_elems=%lld",
                    (long long)chunk_elems, (long long)align_elems);
    if (policy != ELIXIR_LAYOUT_NEXT_FIT && policy != ELIXIR_LAYOUT_FIRST_FIT && policy != ELIXIR_LAYOUT_DENSE)
        return fail(ELIXIR_EINVAL, "elixir_layout_plan: unknown policy %d", policy);
    Planner pl{chunk_elems, align_elems, {}};
    for (int i = 0; i < T; ++i) {
        if (numel[i] < 0) return fail(ELIXIR_EINVAL, "elixir_layout_plan: numel[%d] is negative", i);
        pl.place(numel[i], policy, &chunk_id[i], &offset[i]);
    }
    *n_chunks = (int64_t)pl.used.size();
    if (valid_len) {
        if (valid_cap < *n_chunks)
            return fail(ELIXIR_ECAP, "elixir_layout_plan: valid_len holds %lld entries, %lld chunks planned",
                        (long long)valid_cap, (long long)*n_chunks);
        for (size_t c = 0; c < pl.used.size(); ++c) valid_len[c] = pl.used[c];
    }
    return ELIXIR_OK;
}
}  // namespace

extern "C" int elixir_layout_plan(const int64_t* numel, int T, int64_t chunk_elems, int policy, int64_t align_elems,
                                  int64_t* chunk_id, int64_t* offset, int64_t* n_chunks, int64_t* valid_len,
                                  int64_t valid_cap) {
    return no_throw("elixir_layout_plan", [&] {
        return elixir_layout_plan_impl(numel, T, chunk_elems, policy, align_elems, chunk_id, offset, n_chunks,
                                       valid_len, valid_cap);
    });
}
