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
// The two copy directions run on different streams so that they can use different
// DMA engines (elixir_offload_bind_streams sees to it) and uploads, downloads and
// kernels proceed concurrently.
#include <algorithm>
#include <chrono>
#include <new>
#include <thread>

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

}  // namespace

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
    if (h_block) ELIXIR_HIP_TRY(copy_in_pieces(h_block, sl.d_ptr, bytes, hipMemcpyDeviceToHost, ds));
    ELIXIR_HIP_TRY(hipEventRecord(sl.evicted, ds));
    sl.evict_dst = static_cast<const char*>(h_block);
    sl.evict_bytes = h_block ? bytes : 0;
    sl.evict_pending = true;
    sl.held = false;
    return ELIXIR_OK;
}

// The HIP runtime gives a stream a DMA engine at the stream's first copy (the first engine that is idle at
// that moment) and keeps it.  Two streams whose first copies were issued while nothing else was copying
// therefore share one engine, and uploads and downloads take turns (measured: 28.7 GB/s each way instead of
// 48.6).  Issuing the download stream's first copy while an upload is in flight puts it on another engine.
extern "C" int elixir_offload_bind_streams(elixir_ctx* ctx, elixir_stream_t h2d_stream, elixir_stream_t d2h_stream,
                                           int* overlapped_out) {
    if (!ctx) return fail(ELIXIR_EINVAL, "elixir_offload_bind_streams: ctx is NULL");
    if (overlapped_out) *overlapped_out = 0;
    if (ctx->n_slots == 0) return fail(ELIXIR_ESTATE, "elixir_offload_bind_streams: no staging slots registered");
    if (h2d_stream == d2h_stream) return fail(ELIXIR_EINVAL, "elixir_offload_bind_streams: the two streams are the same");
    for (int i = 0; i < ctx->n_slots; ++i)
        if (ctx->slots[i].held) return fail(ELIXIR_ESTATE, "elixir_offload_bind_streams: slot %d is held", i);
    for (int i = 0; i < ctx->n_slots; ++i)  // slot 0 is about to be overwritten: let pending evictions finish
        if (ctx->slots[i].evict_pending) ELIXIR_HIP_TRY(hipEventSynchronize(ctx->slots[i].evicted));
    hipStream_t up = (hipStream_t)h2d_stream, down = (hipStream_t)d2h_stream;
    // upload into the first half of slot 0, download from its second half
    size_t half = ctx->slot_bytes / 2;
    if (half > ((size_t)128 << 20)) half = (size_t)128 << 20;
    if (half < 4096) return fail(ELIXIR_EINVAL, "elixir_offload_bind_streams: slots of %zu bytes are too small", ctx->slot_bytes);
    char* d = static_cast<char*>(ctx->slots[0].d_ptr);
    char* h = nullptr;
    ELIXIR_HIP_TRY(hipHostMalloc((void**)&h, 2 * half, hipHostMallocDefault));
    auto bail = [&](hipError_t e, const char* what) {
        (void)hipDeviceSynchronize();
        (void)hipHostFree(h);
        return fail(ELIXIR_EHIP, "elixir_offload_bind_streams: %s: %s", what, hipGetErrorString(e));
    };
    hipError_t e;
    // The upload must really be running when the download is issued, not merely queued (the very first copy of a
    // process takes a while to start): wait a quarter of its expected duration, at most half a millisecond.
    const auto head_start = std::chrono::microseconds(std::min<long long>(500, (long long)(half / 200000)));
    auto seconds = [&](bool with_down) -> double {
        const auto t0 = std::chrono::steady_clock::now();
        (void)hipMemcpyAsync(d, h, half, hipMemcpyHostToDevice, up);
        if (with_down) (void)hipMemcpyAsync(h + half, d + half, half, hipMemcpyDeviceToHost, down);
        (void)hipStreamSynchronize(up);
        (void)hipStreamSynchronize(down);
        return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    };
    int overlapped = 0;
    for (int attempt = 0; attempt < 3 && !overlapped; ++attempt) {
        // 1. the latch: the download stream's copy is issued while the upload is running
        if ((e = hipMemcpyAsync(d, h, half, hipMemcpyHostToDevice, up)) != hipSuccess) return bail(e, "upload");
        std::this_thread::sleep_for(head_start);
        if ((e = hipMemcpyAsync(h + half, d + half, half, hipMemcpyDeviceToHost, down)) != hipSuccess) return bail(e, "download");
        if ((e = hipStreamSynchronize(up)) != hipSuccess) return bail(e, "sync");
        if ((e = hipStreamSynchronize(down)) != hipSuccess) return bail(e, "sync");
        // 2. the check: both directions together must take clearly less than the two one after the other
        double t_up = 1e30, t_both = 1e30;  // best of three each: one late wake-up of this thread must not decide
        for (int r = 0; r < 3; ++r) t_up = std::min(t_up, seconds(false));
        for (int r = 0; r < 3; ++r) t_both = std::min(t_both, seconds(true));
        if ((e = hipGetLastError()) != hipSuccess) return bail(e, "timed copies");
        overlapped = t_both < 1.6 * t_up ? 1 : 0;
    }
    if (overlapped_out) *overlapped_out = overlapped;
    ELIXIR_HIP_TRY(hipHostFree(h));
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
