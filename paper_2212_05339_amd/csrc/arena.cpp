// Placement of the long-lived chunk buffers inside allocations the caller makes once, before training (host only,
// integers, no allocation).
//
// The paper allocates what lives as long as the training run -- optimizer states, rCache blocks -- before training
// starts (Sec. 3, "Pre-runtime Profiler", finding 2).  Where those buffers lie relative to each other decides a few
// percent of the update's bandwidth on MI355X, measured on whole 64Mi-element launches:
//   * the arrays one kernel reads together (a chunk's optimizer chunk, its gradient arrays, its fp32 gradient chunk)
//     want to lie side by side in one allocation: the AdamW launch takes 266-270 us with the gradient array next to
//     the optimizer chunk and 280-283 us with it tens of GiB away; the accumulate pass of the reduction 99-102 us
//     against 106-109 us;
//   * arrays that are only written (the low-precision parameter copies) want to lie somewhere else (2%);
//   * arrays whose starts are a multiple of a few MiB apart make the kernel's streams cross DRAM pages in phase
//     (2%): every array is followed by a gap of 4 MiB + 8 KiB.
// elixir_arena_plan turns a description of the arrays of one chunk into byte offsets: the NEAR arrays chunk after
// chunk in one region, the FAR arrays chunk after chunk in another; the caller allocates the two regions (as far
// apart as it can) and carves the buffers out of them.
#include "status.hpp"

using namespace elixir;

namespace {
constexpr int64_t kGrain = 8192;  // every array starts on a multiple of this
int64_t slot_bytes(int64_t bytes) { return (bytes + kGrain - 1) / kGrain * kGrain + ELIXIR_ARENA_GAP_BYTES; }
}  // namespace

extern "C" int elixir_arena_plan(int n_chunks, const elixir_arena_array* arrays, int n_arrays, int64_t* offset_out,
                                 int64_t offset_cap, int64_t* region_bytes_out) {
    static const char* what = "elixir_arena_plan";
    if (n_chunks < 0 || n_arrays < 0) return fail(ELIXIR_EINVAL, "%s: negative n_chunks or n_arrays", what);
    if (!region_bytes_out || (n_arrays > 0 && !arrays)) return fail(ELIXIR_EINVAL, "%s: NULL argument", what);
    int64_t per_chunk = 0, group[2] = {0, 0};
    for (int a = 0; a < n_arrays; ++a) {
        const elixir_arena_array& x = arrays[a];
        if (x.bytes < 0 || x.count < 0) return fail(ELIXIR_EINVAL, "%s: array %d has a negative size or count", what, a);
        if (x.region != ELIXIR_ARENA_NEAR && x.region != ELIXIR_ARENA_FAR)
            return fail(ELIXIR_EINVAL, "%s: array %d: region=%d is neither ELIXIR_ARENA_NEAR nor ELIXIR_ARENA_FAR", what, a, x.region);
        if (x.bytes > (INT64_MAX >> 12) || x.count > (1 << 20)) return fail(ELIXIR_ECAP, "%s: array %d is too large", what, a);
        per_chunk += x.count;
        group[x.region] += slot_bytes(x.bytes) * x.count;
        if (group[x.region] > (INT64_MAX >> 24)) return fail(ELIXIR_ECAP, "%s: a chunk's arrays exceed what an allocation can hold", what);
    }
    region_bytes_out[0] = group[0] * n_chunks;
    region_bytes_out[1] = group[1] * n_chunks;
    const int64_t need = per_chunk * n_chunks;
    if (need > offset_cap) return fail(ELIXIR_ECAP, "%s: %lld offsets, offset_out holds %lld", what, (long long)need, (long long)offset_cap);
    if (need > 0 && !offset_out) return fail(ELIXIR_EINVAL, "%s: offset_out is NULL", what);
    int64_t k = 0;
    for (int c = 0; c < n_chunks; ++c) {
        int64_t at[2] = {group[0] * c, group[1] * c};
        for (int a = 0; a < n_arrays; ++a) {
            const elixir_arena_array& x = arrays[a];
            for (int j = 0; j < x.count; ++j) {
                offset_out[k++] = at[x.region];
                at[x.region] += slot_bytes(x.bytes);
            }
        }
    }
    return ELIXIR_OK;
}
