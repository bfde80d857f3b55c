// rCache replacement simulation and the chunk-size search built on it (host only, integers).
//
// The paper keeps gathered chunks in an rCache of n_block equal blocks and, because the order in which
// chunks are used is known before training, replaces them with Belady's rule: evict the chunk whose next
// use lies farthest ahead (Sec. 3 "rCache").  The chunk length is chosen by simulating candidate lengths
// and taking the one with the fewest bytes replaced in the rCache during one training step (App. A.2;
// the paper does this simulation in C++ as well).  One step uses the parameters in their forward order
// and then in the reverse order (Sec. 5.1: the backward pass calls parameters in exactly the reverse order).
#include <queue>
#include <utility>
#include <vector>

#include "status.hpp"

using namespace elixir;

namespace {

const int64_t kNever = INT64_MAX;

// Belady replay.  next[i] = position of the next access to seq[i] after i, or kNever.
void replay(const std::vector<int64_t>& seq, int64_t n_ids, int64_t n_blocks, int64_t* misses, int64_t* evictions) {
    const int64_t len = (int64_t)seq.size();
    std::vector<int64_t> next(len), last(n_ids, kNever);
    for (int64_t i = len - 1; i >= 0; --i) {
        next[i] = last[seq[i]];
        last[seq[i]] = i;
    }
    // cached[id] = position of its next use while cached, -1 when not cached.  The heap holds (next use, -id) so
    // that the farthest next use comes first and, among chunks never used again, the lowest id; stale entries
    // (whose next-use value no longer matches) are skipped when popped.
    std::vector<int64_t> cached(n_ids, -1);
    std::priority_queue<std::pair<int64_t, int64_t>> heap;
    int64_t in_cache = 0, m = 0, e = 0;
    for (int64_t i = 0; i < len; ++i) {
        const int64_t id = seq[i];
        if (cached[id] < 0) {
            ++m;
            if (in_cache == n_blocks) {
                for (;;) {
                    const auto top = heap.top();
                    heap.pop();
                    const int64_t victim = -top.second;
                    if (cached[victim] == top.first) {
                        cached[victim] = -1;
                        break;
                    }
                }
                ++e;
                --in_cache;
            }
            ++in_cache;
        }
        cached[id] = next[i];
        heap.push({next[i], -id});
    }
    *misses = m;
    *evictions = e;
}

int elixir_rcache_simulate_impl(const int64_t* seq, int64_t len, int64_t n_blocks, int64_t* misses_out,
                                int64_t* evictions_out) {
    static const char* what = "elixir_rcache_simulate";
    if (len < 0 || (len > 0 && !seq) || !misses_out || !evictions_out) return fail(ELIXIR_EINVAL, "%s: bad arguments", what);
    if (n_blocks < 1) return fail(ELIXIR_EINVAL, "%s: n_blocks=%lld, at least one block is needed", what, (long long)n_blocks);
    int64_t max_id = -1;
    for (int64_t i = 0; i < len; ++i) {
        if (seq[i] < 0) return fail(ELIXIR_EINVAL, "%s: seq[%lld] is negative", what, (long long)i);
        if (seq[i] > max_id) max_id = seq[i];
    }
    if (max_id > 4 * len + 1024) return fail(ELIXIR_EINVAL, "%s: chunk ids are not dense (largest id %lld)", what, (long long)max_id);
    std::vector<int64_t> s(seq, seq + len);
    replay(s, max_id + 1, n_blocks, misses_out, evictions_out);
    return ELIXIR_OK;
}
}  // namespace

extern "C" int elixir_rcache_simulate(const int64_t* seq, int64_t len, int64_t n_blocks, int64_t* misses_out,
                                      int64_t* evictions_out) {
    return no_throw("elixir_rcache_simulate", [&] {
        return elixir_rcache_simulate_impl(seq, len, n_blocks, misses_out, evictions_out);
    });
}

namespace {
int elixir_chunk_size_search_impl(const int64_t* numel, int T, const int64_t* candidates, int n_cand, int policy,
                                  int64_t align_elems, double cache_bytes, int L_c, int* best_out,
                                  int64_t* replaced_bytes_out, int64_t* padding_out) {
    static const char* what = "elixir_chunk_size_search";
    if (T < 0 || n_cand < 1 || !candidates || !best_out || !replaced_bytes_out || (T > 0 && !numel))
        return fail(ELIXIR_EINVAL, "%s: bad arguments", what);
    if (L_c < 1 || !(cache_bytes >= 0)) return fail(ELIXIR_EINVAL, "%s: L_c must be positive and cache_bytes non-negative", what);
    std::vector<int64_t> cid(T > 0 ? T : 1), off(T > 0 ? T : 1);
    int best = -1;
    int64_t best_replaced = 0, best_padding = 0;
    for (int k = 0; k < n_cand; ++k) {
        const int64_t C = candidates[k];
        int64_t n_chunks = 0;
        if (const int rc = elixir_layout_plan(numel, T, C, policy, align_elems, cid.data(), off.data(), &n_chunks, nullptr, 0)) return rc;
        // one training step: every parameter in forward order, then in reverse; a parameter touches every chunk it
        // spans; consecutive accesses to the same chunk are one access
        std::vector<int64_t> seq;
        auto touch = [&](int64_t c) {
            if (seq.empty() || seq.back() != c) seq.push_back(c);
        };
        int64_t used = 0;
        for (int i = 0; i < T; ++i) {
            used += numel[i];
            if (numel[i] == 0) continue;
            const int64_t first = cid[i], last = cid[i] + (off[i] + numel[i] - 1) / C;
            for (int64_t c = first; c <= last; ++c) touch(c);
        }
        for (int i = T - 1; i >= 0; --i) {
            if (numel[i] == 0) continue;
            const int64_t first = cid[i], last = cid[i] + (off[i] + numel[i] - 1) / C;
            for (int64_t c = last; c >= first; --c) touch(c);
        }
        int64_t blocks = (int64_t)(cache_bytes / ((double)L_c * (double)C));
        if (blocks < 1) blocks = 1;
        int64_t misses = 0, evictions = 0;
        replay(seq, n_chunks > 0 ? n_chunks : 1, blocks, &misses, &evictions);
        const int64_t replaced = evictions * (int64_t)L_c * C;
        const int64_t padding = n_chunks * C - used;
        replaced_bytes_out[k] = replaced;
        if (padding_out) padding_out[k] = padding;
        // fewest replaced bytes; then least padding; then the longer chunk (fewer, larger transfers)
        if (best < 0 || replaced < best_replaced || (replaced == best_replaced && padding < best_padding) ||
            (replaced == best_replaced && padding == best_padding && C > candidates[best])) {
            best = k;
            best_replaced = replaced;
            best_padding = padding;
        }
    }
    *best_out = best;
    return ELIXIR_OK;
}
}  // namespace

extern "C" int elixir_chunk_size_search(const int64_t* numel, int T, const int64_t* candidates, int n_cand, int policy,
                                        int64_t align_elems, double cache_bytes, int L_c, int* best_out,
                                        int64_t* replaced_bytes_out, int64_t* padding_out) {
    return no_throw("elixir_chunk_size_search", [&] {
        return elixir_chunk_size_search_impl(numel, T, candidates, n_cand, policy, align_elems, cache_bytes, L_c,
                                             best_out, replaced_bytes_out, padding_out);
    });
}
