// Offload pipeline: staging slots, prefetch (host -> device) and evict (device -> host)
// of host-resident optimizer chunks on side streams.
//
// The paper overlaps chunk movement with computation by issuing it on separate
// streams in the known order of use (Sec. 4.3).  Here ordering is expressed
// only with events, so the host thread never blocks:
//   prefetch : h2d stream waits for the slot's previous eviction and for any pending eviction into the host block
//              it is about to read, copies, records `ready`
//   wait     : compute stream waits for `ready`
//   evict    : d2h stream waits for an event recorded on the compute stream,
//              copies back, records `evicted`
// The two copy directions and the updates run on three streams so that uploads, downloads and
// kernels proceed concurrently; elixir_offload_copy_streams provides copy streams for which that is
// measured to hold.
#include <stdlib.h>

#include <algorithm>
#include <chrono>
#include <mutex>
#include <new>

#include "common.hpp"

namespace elixir {
void destroy_slots(elixir_ctx* c);
}
using namespace elixir;

namespace {

// Block copies are issued in pieces: a DMA engine serves the streams that share it one command at a time, so a
// 1.6 GB command would make a small copy on another stream (the gradients of a CPU-updated chunk) wait 30 ms.
constexpr size_t kDmaPiece = (size_t)256 << 20;

hipError_t copy_in_pieces(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t s) {
    char* d = static_cast<char*>(dst);
    const char* q = static_cast<const char*>(src);
    while (bytes > 0) {
        const size_t n = bytes < kDmaPiece ? bytes : kDmaPiece;
        const hipError_t e = hipMemcpyAsync(d, q, n, kind, s);
        if (e != hipSuccess) return e;
        d += n;
        q += n;
        bytes -= n;
    }
    return hipSuccess;
}

// The download of a slot by a kernel instead of the DMA engine: every lane stores 16 bytes into the pinned block, the
// stores travel over the link as posted writes.  Meant for a process in which uploads and downloads by DMA take turns
// (see elixir_offload_copy_streams below): the upload keeps its DMA engine, the download no longer competes for one.
// A fixed, small grid with a stride loop: the link, not the chip, bounds the copy (16 to 1024 workgroups measure the same,
// 8 are too few), and the compute stream's kernels keep most of the compute units.  Every thread's loop ends at n16, so
// the grid always drains.  Measured in the pipeline with 12 blocks of 805 MB: 42.5-46.9 GB/s each way from box to box
// where the DMA engine gives 45.9, and the same 42.5-46.9 where the DMA engines take turns and give 27.6-34.0.
constexpr int kStoreBlocks = 64;
constexpr int kStoreThreads = 256;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kStoreThreads) void host_store_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16,
                                                                  int tail_bytes) {
    const int64_t stride = (int64_t)gridDim.x * kStoreThreads;
    for (int64_t i = (int64_t)blockIdx.x * kStoreThreads + threadIdx.x; i < n16; i += stride) dst[i] = __builtin_nontemporal_load(src + i);
    if (blockIdx.x == 0 && (int)threadIdx.x < tail_bytes)  // the last bytes of a length that is no multiple of 16
        reinterpret_cast<char*>(dst + n16)[threadIdx.x] = reinterpret_cast<const char*>(src + n16)[threadIdx.x];
}

// The address under which the device reaches [h, h + bytes) of pinned host memory, or nullptr if that cannot be shown
// (pageable memory, a range that leaves its allocation): the caller then copies by DMA, which needs no such address.
char* device_view_of_pinned(void* h, size_t bytes) {
    hipPointerAttribute_t a0, a1;
    if (hipPointerGetAttributes(&a0, h) != hipSuccess || hipPointerGetAttributes(&a1, static_cast<char*>(h) + bytes - 1) != hipSuccess) {
        (void)hipGetLastError();  // a pointer the runtime does not know is no error of this call
        return nullptr;
    }
    if (a0.type != hipMemoryTypeHost || a1.type != hipMemoryTypeHost || !a0.devicePointer || !a1.devicePointer) return nullptr;
    if (static_cast<char*>(a1.devicePointer) - static_cast<char*>(a0.devicePointer) != (ptrdiff_t)(bytes - 1)) return nullptr;
    return static_cast<char*>(a0.devicePointer);
}

}  // namespace

extern "C" int elixir_offload_set_evict_path(elixir_ctx* ctx, int path) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_offload_set_evict_path: ctx is NULL");
    if (path != ELIXIR_EVICT_DMA && path != ELIXIR_EVICT_KERNEL)
        return fail(ELIXIR_EINVAL, "elixir_offload_set_evict_path: path=%d is neither ELIXIR_EVICT_DMA nor ELIXIR_EVICT_KERNEL", path);
    ctx->evict_path = path;
    return ELIXIR_OK;
}

extern "C" int elixir_offload_register_slots(elixir_ctx* ctx, void* const* d_slots, int n_slots, size_t slot_bytes) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_offload_register_slots: ctx is NULL");
    if (n_slots < 0 || (n_slots > 0 && (!d_slots || slot_bytes == 0)))
        return fail(ELIXIR_EINVAL, "elixir_offload_register_slots: bad slot table");
    for (int i = 0; i < ctx->n_slots; ++i)
        if (ctx->slots[i].held) return fail(ELIXIR_ESTATE, "elixir_offload_register_slots: slot %d is still held", i);
    for (int i = 0; i < n_slots; ++i)
        if (!d_slots[i]) return fail(ELIXIR_EINVAL, "elixir_offload_register_slots: d_slots[%d] is NULL", i);
    // pending evictions of the old registration must have finished before their events go away
    for (int i = 0; i < ctx->n_slots; ++i)
        if (ctx->slots[i].evict_pending) ELIXIR_HIP_TRY(hipEventSynchronize(ctx->slots[i].evicted));
    destroy_slots(ctx);
    if (n_slots == 0) return ELIXIR_OK;
    ctx->slots = new (std::nothrow) Slot[n_slots];
    if (!ctx->slots) return fail(ELIXIR_EINVAL, "elixir_offload_register_slots: out of host memory");
    ctx->n_slots = n_slots;
    ctx->slot_bytes = slot_bytes;
    for (int i = 0; i < n_slots; ++i) {
        ctx->slots[i].d_ptr = d_slots[i];
        hipError_t e = hipEventCreateWithFlags(&ctx->slots[i].ready, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->slots[i].updated, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->slots[i].evicted, hipEventDisableTiming);
        if (e != hipSuccess) {
            destroy_slots(ctx);
            return fail(ELIXIR_EHIP, "elixir_offload_register_slots: hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    return ELIXIR_OK;
}

extern "C" int elixir_chunk_prefetch(elixir_ctx* ctx, const void* h_block, size_t bytes, int* slot_out,
                                     elixir_stream_t h2d_stream) {
    if (!ctx || !h_block || !slot_out) return fail(ELIXIR_EINVAL, "elixir_chunk_prefetch: NULL argument");
    if (ctx->n_slots == 0) return fail(ELIXIR_ESTATE, "elixir_chunk_prefetch: no staging slots registered");
    if (bytes == 0 || bytes > ctx->slot_bytes)
        return fail(ELIXIR_EINVAL, "elixir_chunk_prefetch: %zu bytes, slots hold %zu", bytes, ctx->slot_bytes);
    int slot = -1;
    for (int k = 0; k < ctx->n_slots; ++k) {  // round robin: the slot evicted longest ago comes first
        const int i = (ctx->next_slot + k) % ctx->n_slots;
        if (!ctx->slots[i].held) { slot = i; break; }
    }
    if (slot < 0) return fail(ELIXIR_ENOSLOT, "elixir_chunk_prefetch: all %d slots are held", ctx->n_slots);
    Slot& sl = ctx->slots[slot];
    hipStream_t s = (hipStream_t)h2d_stream;
    if (sl.evict_pending) ELIXIR_HIP_TRY(hipStreamWaitEvent(s, sl.evicted, 0));
    // The host block may still be the target of an eviction from ANOTHER slot (few host chunks, slots taken round
    // robin: a block evicted from slot 0 comes back through slot 1): the upload must not read it before that
    // download has landed.
    const char* src = static_cast<const char*>(h_block);
    for (int i = 0; i < ctx->n_slots; ++i) {
        const Slot& o = ctx->slots[i];
        if (i == slot || !o.evict_pending || !o.evict_dst) continue;
        if (src < o.evict_dst + o.evict_bytes && o.evict_dst < src + bytes) ELIXIR_HIP_TRY(hipStreamWaitEvent(s, o.evicted, 0));
    }
    ELIXIR_HIP_TRY(copy_in_pieces(sl.d_ptr, h_block, bytes, hipMemcpyHostToDevice, s));
    ELIXIR_HIP_TRY(hipEventRecord(sl.ready, s));
    sl.held = true;
    ctx->next_slot = (slot + 1) % ctx->n_slots;
    *slot_out = slot;
    return ELIXIR_OK;
}

extern "C" int elixir_chunk_wait_ready(elixir_ctx* ctx, int slot, elixir_stream_t compute_stream) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_chunk_wait_ready: ctx is NULL");
    if (slot < 0 || slot >= ctx->n_slots) return fail(ELIXIR_EINVAL, "elixir_chunk_wait_ready: slot %d of %d", slot, ctx->n_slots);
    if (!ctx->slots[slot].held) return fail(ELIXIR_ESTATE, "elixir_chunk_wait_ready: slot %d holds no prefetched chunk", slot);
    ELIXIR_HIP_TRY(hipStreamWaitEvent((hipStream_t)compute_stream, ctx->slots[slot].ready, 0));
    return ELIXIR_OK;
}

extern "C" int elixir_chunk_evict(elixir_ctx* ctx, int slot, void* h_block, size_t bytes, elixir_stream_t compute_stream,
                                  elixir_stream_t d2h_stream) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_chunk_evict: ctx is NULL");
    if (slot < 0 || slot >= ctx->n_slots) return fail(ELIXIR_EINVAL, "elixir_chunk_evict: slot %d of %d", slot, ctx->n_slots);
    Slot& sl = ctx->slots[slot];
    if (!sl.held) return fail(ELIXIR_ESTATE, "elixir_chunk_evict: slot %d holds no prefetched chunk", slot);
    if (h_block && (bytes == 0 || bytes > ctx->slot_bytes))
        return fail(ELIXIR_EINVAL, "elixir_chunk_evict: %zu bytes, slots hold %zu", bytes, ctx->slot_bytes);
    hipStream_t cs = (hipStream_t)compute_stream, ds = (hipStream_t)d2h_stream;
    // everything enqueued so far on the compute stream (the update of this slot) must finish first
    ELIXIR_HIP_TRY(hipEventRecord(sl.updated, cs));
    ELIXIR_HIP_TRY(hipStreamWaitEvent(ds, sl.updated, 0));
    if (h_block) {
        char* dview = nullptr;
        if (ctx->evict_path == ELIXIR_EVICT_KERNEL && aligned(sl.d_ptr, 16)) dview = device_view_of_pinned(h_block, bytes);
        if (dview && aligned(dview, 16)) {
            hipLaunchKernelGGL(host_store_kernel, dim3(kStoreBlocks), dim3(kStoreThreads), 0, ds, static_cast<const u32x4*>(sl.d_ptr),
                               reinterpret_cast<u32x4*>(dview), (int64_t)(bytes / 16), (int)(bytes % 16));
            ELIXIR_HIP_TRY(hipGetLastError());
        } else {
            ELIXIR_HIP_TRY(copy_in_pieces(h_block, sl.d_ptr, bytes, hipMemcpyDeviceToHost, ds));
        }
    }
    ELIXIR_HIP_TRY(hipEventRecord(sl.evicted, ds));
    sl.evict_dst = static_cast<const char*>(h_block);
    sl.evict_bytes = h_block ? bytes : 0;
    sl.evict_pending = true;
    sl.held = false;
    return ELIXIR_OK;
}

// Copy streams that really run beside the compute stream.
//
// The HIP runtime feeds all streams of a process through a few hardware queues (GPU_MAX_HW_QUEUES, 4 by default): a
// new stream joins the queue with the fewest streams on it.  Two streams on one hardware queue are still ordered
// correctly, but a wait that one of them has queued (hipStreamWaitEvent, the marker behind a copy) holds back whatever
// the other one queues behind it.  Measured on MI355X with the offload pipeline of this file: upload and download
// streams on one queue take turns (28 GB/s each way instead of 46-48), and a compute stream that shares a queue with
// a copy stream has its kernels wait for 30 ms block copies.  Which streams share a queue depends on how many streams
// the process has created before (seen: 1 or 2 streams created earlier break the pipeline, 0, 3, 5, 9 or 14 do not), so
// it cannot be arranged by construction; it can be measured: a marker on stream B that completes only when a long copy
// on stream A has finished shares A's queue.  elixir_offload_copy_streams creates candidate streams until it has two
// that share a queue neither with the caller's compute stream nor with each other.
//
// Separate queues are necessary, not sufficient.  After device memory has been freed, downloads by DMA run at half rate
// for a while (a download alone 30 GB/s instead of 57, an upload and a download together 29 GB/s each way instead of
// 48.6; uploads alone are not affected): about 30 ms per GiB freed, whatever is copied meanwhile (measured: 16 GiB
// under 0.5 s, 64 GiB 2 s), also after the exit of an earlier process on the same GPU.  hipFree itself returns at
// once, so this looks like work the driver does on the freed memory with the engine that serves downloads.  No stream
// choice changes it, so the call only reports it: *full_duplex_out says whether an upload and a download overlapped
// when the call looked.  A process that wants the full-duplex rate allocates its long-lived buffers once and frees
// nothing large while it streams (the paper's own rule for long-lived buffers, Sec. 3 "Pre-runtime Profiler"); one
// that cannot wait lets the slots come back by the store kernel above (elixir_offload_set_evict_path), which needs no
// DMA engine.

namespace {

struct QueueProbe {
    char* d_buf = nullptr;
    char* h_buf = nullptr;
    size_t bytes = (size_t)64 << 20;  // ~1.1 ms on the link: far above the ~20 us an unhindered marker takes (buffers hold two such pieces)
    hipEvent_t ea = nullptr, eb = nullptr;
    bool verbose = getenv("ELIXIR_TRACE_STREAMS") != nullptr;  // prints what was measured for every candidate
    ~QueueProbe() {
        if (ea) (void)hipEventDestroy(ea);
        if (eb) (void)hipEventDestroy(eb);
        if (d_buf) (void)hipFree(d_buf);
        if (h_buf) (void)hipHostFree(h_buf);
    }
    hipError_t init() {
        hipError_t e = hipMalloc((void**)&d_buf, 2 * bytes);
        if (e == hipSuccess) e = hipHostMalloc((void**)&h_buf, 2 * bytes, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ea, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&eb, hipEventDisableTiming);
        return e;
    }
    // *shared = a marker on b waits for the work pending on a.  Best of three: a late wake-up of this thread can only
    // make an independent pair look dependent, never the other way round.
    hipError_t shares_queue(hipStream_t a, hipStream_t b, bool* shared) {
        double best = 1e30;
        for (int r = 0; r < 3 && best > 0.25; ++r) {
            hipError_t e = hipMemcpyAsync(d_buf, h_buf, bytes, hipMemcpyHostToDevice, a);
            if (e == hipSuccess) e = hipEventRecord(ea, a);
            const auto t0 = std::chrono::steady_clock::now();
            if (e == hipSuccess) e = hipEventRecord(eb, b);
            if (e == hipSuccess) e = hipEventSynchronize(eb);
            const auto t1 = std::chrono::steady_clock::now();
            if (e == hipSuccess) e = hipEventSynchronize(ea);
            const auto t2 = std::chrono::steady_clock::now();
            if (e != hipSuccess) {
                (void)hipDeviceSynchronize();
                return e;
            }
            const double marker = std::chrono::duration<double>(t1 - t0).count(), copy = std::chrono::duration<double>(t2 - t0).count();
            best = std::min(best, marker / copy);
        }
        *shared = best > 0.5;
        if (verbose) fprintf(stderr, "elixir_offload_copy_streams: marker on %p behind a copy on %p: %.0f%% of the copy's time -> %s\n", (void*)b,
                             (void*)a, 100.0 * best, *shared ? "same hardware queue" : "independent");
        return hipSuccess;
    }
    // *overlap = an upload on `up` and a download on `down` issued together take clearly less than the two one after the
    // other.  The runtime picks a DMA engine for a copy from those that are idle when the copy is issued, so the
    // first download is issued while an upload is known to be running (a small upload and a marker in front of a long
    // one: once the marker has completed the engine is working on the long one).  Best of three each.
    hipError_t copies_overlap(hipStream_t up, hipStream_t down, bool* overlap) {
        hipError_t e = hipMemcpyAsync(d_buf, h_buf, 4096, hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipEventRecord(ea, up);
        if (e == hipSuccess) e = hipMemcpyAsync(d_buf, h_buf, bytes, hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipEventSynchronize(ea);
        if (e == hipSuccess) e = hipMemcpyAsync(h_buf + bytes, d_buf + bytes, bytes, hipMemcpyDeviceToHost, down);
        if (e == hipSuccess) e = hipStreamSynchronize(up);
        if (e == hipSuccess) e = hipStreamSynchronize(down);
        double t_up = 1e30, t_both = 1e30;
        for (int r = 0; r < 6 && e == hipSuccess; ++r) {
            const bool both = r >= 3;
            const auto t0 = std::chrono::steady_clock::now();
            e = hipMemcpyAsync(d_buf, h_buf, bytes, hipMemcpyHostToDevice, up);
            if (both && e == hipSuccess) e = hipMemcpyAsync(h_buf + bytes, d_buf + bytes, bytes, hipMemcpyDeviceToHost, down);
            if (e == hipSuccess) e = hipStreamSynchronize(up);
            if (e == hipSuccess) e = hipStreamSynchronize(down);
            const double t = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
            if (both) t_both = std::min(t_both, t);
            else t_up = std::min(t_up, t);
        }
        if (e != hipSuccess) {
            (void)hipDeviceSynchronize();
            return e;
        }
        *overlap = t_both < 1.6 * t_up;
        if (verbose) fprintf(stderr, "elixir_offload_copy_streams: upload on %p %.3f ms, with a download on %p %.3f ms -> %s\n", (void*)up,
                             1e3 * t_up, (void*)down, 1e3 * t_both, *overlap ? "they overlap" : "they take turns");
        return hipSuccess;
    }
};

}  // namespace

namespace {
// The pair is kept per device for the life of the process and each stream keeps its direction: a stream that is
// destroyed hands its hardware queue, and with it the DMA engine it used, to the next stream created, and an
// engine picked for downloads was then seen to serve uploads at half the link rate.
constexpr int kMaxDevices = 64;
std::mutex g_pair_mutex;
hipStream_t g_pair[kMaxDevices][2] = {};
}  // namespace

extern "C" int elixir_offload_copy_streams(elixir_ctx* ctx, elixir_stream_t compute_stream, elixir_stream_t* h2d_out,
                                           elixir_stream_t* d2h_out, int* full_duplex_out) {
    static const char* what = "elixir_offload_copy_streams";
    if (!ctx || !h2d_out || !d2h_out) return fail(ELIXIR_EINVAL, "%s: NULL argument", what);
    *h2d_out = *d2h_out = nullptr;
    if (full_duplex_out) *full_duplex_out = 0;
    if (ctx->device < 0 || ctx->device >= kMaxDevices) return fail(ELIXIR_ECAP, "%s: device %d", what, ctx->device);
    std::lock_guard<std::mutex> lock(g_pair_mutex);
    QueueProbe probe;
    hipError_t e = probe.init();
    if (e != hipSuccess) return fail(ELIXIR_EHIP, "%s: set-up of the probe: %s", what, hipGetErrorString(e));
    hipStream_t cs = (hipStream_t)compute_stream;
    hipStream_t* pair = g_pair[ctx->device];
    // does the pair this process already has still run beside this compute stream?
    if (pair[0] && pair[1]) {
        bool up_shared = true, down_shared = true, each_other = true, overlap = false;
        e = probe.shares_queue(cs, pair[0], &up_shared);
        if (e == hipSuccess) e = probe.shares_queue(cs, pair[1], &down_shared);
        if (e == hipSuccess) e = probe.shares_queue(pair[0], pair[1], &each_other);
        if (e == hipSuccess && !up_shared && !down_shared && !each_other) e = probe.copies_overlap(pair[0], pair[1], &overlap);
        if (e != hipSuccess) return fail(ELIXIR_EHIP, "%s: probing the existing streams: %s", what, hipGetErrorString(e));
        if (!up_shared && !down_shared && !each_other) {
            *h2d_out = pair[0];
            *d2h_out = pair[1];
            if (full_duplex_out) *full_duplex_out = overlap ? 1 : 0;
            return ELIXIR_OK;
        }
        // Not beside this compute stream: a new pair is looked for.  The old one is left alone (a pipeline may still use it).
        pair[0] = pair[1] = nullptr;
    }
    // Candidates stay alive until the end: each one raises the stream count of its hardware queue, which is what sends
    // the next candidate to another queue.
    constexpr int kCandidates = 12;
    hipStream_t cand[kCandidates] = {};
    hipStream_t kept[2] = {nullptr, nullptr};
    int n_cand = 0, n_kept = 0;
    int rc = ELIXIR_OK;
    for (; n_cand < kCandidates && n_kept < 2; ++n_cand) {
        if ((e = hipStreamCreateWithFlags(&cand[n_cand], hipStreamNonBlocking)) != hipSuccess) {
            rc = fail(ELIXIR_EHIP, "%s: hipStreamCreateWithFlags: %s", what, hipGetErrorString(e));
            break;
        }
        hipStream_t s = cand[n_cand];
        bool shared = false;
        if ((e = probe.shares_queue(cs, s, &shared)) == hipSuccess && !shared && n_kept == 1) e = probe.shares_queue(kept[0], s, &shared);
        if (e != hipSuccess) {
            rc = fail(ELIXIR_EHIP, "%s: probing a stream: %s", what, hipGetErrorString(e));
            ++n_cand;
            break;
        }
        if (!shared) kept[n_kept++] = s;
    }
    for (int i = 0; i < n_cand; ++i)
        if (cand[i] && cand[i] != kept[0] && cand[i] != kept[1]) (void)hipStreamDestroy(cand[i]);
    if (rc == ELIXIR_OK && n_kept < 2)
        rc = fail(ELIXIR_ESTATE, "%s: of %d new streams fewer than two have a hardware queue to themselves beside the compute stream", what, n_cand);
    bool overlap = false;
    if (rc == ELIXIR_OK && (e = probe.copies_overlap(kept[0], kept[1], &overlap)) != hipSuccess)
        rc = fail(ELIXIR_EHIP, "%s: probing the copies: %s", what, hipGetErrorString(e));
    if (rc != ELIXIR_OK) {
        for (hipStream_t k : kept)
            if (k) (void)hipStreamDestroy(k);
        return rc;
    }
    pair[0] = kept[0];
    pair[1] = kept[1];
    *h2d_out = kept[0];
    *d2h_out = kept[1];
    if (full_duplex_out) *full_duplex_out = overlap ? 1 : 0;
    return ELIXIR_OK;
}

// Plain asynchronous copies between pinned host memory and device memory on the caller's stream: what the
// CPU-update path needs (low-precision gradients down, low-precision parameters up).
extern "C" int elixir_copy_h2d_async(void* d_dst, const void* h_src, size_t bytes, elixir_stream_t stream) {
    if (bytes == 0) return ELIXIR_OK;
    if (!d_dst || !h_src) return fail(ELIXIR_EINVAL, "elixir_copy_h2d_async: NULL pointer");
    ELIXIR_HIP_TRY(hipMemcpyAsync(d_dst, h_src, bytes, hipMemcpyHostToDevice, (hipStream_t)stream));
    return ELIXIR_OK;
}

extern "C" int elixir_copy_d2h_async(void* h_dst, const void* d_src, size_t bytes, elixir_stream_t stream) {
    if (bytes == 0) return ELIXIR_OK;
    if (!h_dst || !d_src) return fail(ELIXIR_EINVAL, "elixir_copy_d2h_async: NULL pointer");
    ELIXIR_HIP_TRY(hipMemcpyAsync(h_dst, d_src, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream));
    return ELIXIR_OK;
}

extern "C" int elixir_stream_synchronize(elixir_stream_t stream) {
    ELIXIR_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return ELIXIR_OK;
}
