// Internal helpers shared by the translation units of libelixir_chunk.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>

#include "../../include/elixir_chunk.h"

#include "status.hpp"

namespace elixir {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

#define ELIXIR_HIP_TRY(expr)                                                                         \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess) {                                                                      \
            (void)hipGetLastError(); /* reported here; do not leave it for the caller's next HIP call */ \
            return ::elixir::fail(ELIXIR_EHIP, "%s: %s", #expr, hipGetErrorString(e_));             \
        }                                                                                            \
    } while (0)

// Launch check: hipGetLastError after a kernel launch.
#define ELIXIR_LAUNCH_CHECK(what)                                                                    \
    do {                                                                                             \
        hipError_t e_ = hipGetLastError();                                                           \
        if (e_ != hipSuccess) return ::elixir::fail(ELIXIR_EHIP, "launch of %s: %s", what, hipGetErrorString(e_)); \
    } while (0)

constexpr int kNormBlocksPerChunk = 1024;  // fixed, so the reduction tree never depends on the launch

int norm_scratch_init();  // norm.hip: looks up the static norm workspace of the current device (idempotent)

struct Slot {
    void* d_ptr = nullptr;
    bool held = false;          // prefetched and not yet evicted
    bool evict_pending = false; // an eviction was enqueued; evicted event is valid
    hipEvent_t ready = nullptr;   // H2D copy finished
    hipEvent_t updated = nullptr; // compute stream reached the eviction request
    hipEvent_t evicted = nullptr; // D2H copy finished (slot reusable)
    const char* evict_dst = nullptr;  // host range the last eviction writes (valid while evict_pending)
    size_t evict_bytes = 0;
};

}  // namespace elixir

struct elixir_ctx {
    int device = 0;
    int64_t max_chunk_elems = 0;
    int max_chunks = 0;
    double* d_partials = nullptr;  // max_chunks * kNormBlocksPerChunk
    double* d_stage = nullptr;     // one double per wavefront of the fused reduce + sum-of-squares pass (one chunk at a time)
    int64_t stage_len = 0;
    elixir::Slot* slots = nullptr;
    int n_slots = 0;
    size_t slot_bytes = 0;
    int next_slot = 0;
    int evict_path = 0;            // ELIXIR_EVICT_DMA or ELIXIR_EVICT_KERNEL (offload.cpp)
    // the fused reduction + sum-of-squares calls of one step share d_stage and d_partials: they must arrive on one stream
    bool fused_open = false;       // a sumsq call has been made since the last finish
    void* fused_stream = nullptr;  // the stream of that call
};
