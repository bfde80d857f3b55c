// Context life cycle, error reporting, pinned host memory.
#include <stdarg.h>

#include <new>

#include "common.hpp"

namespace elixir {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Makes `device` current for the lifetime of the guard and restores the previous one.
struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int device) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == device) || hipSetDevice(device) == hipSuccess;
        if (prev == device) prev = -1;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

}  // namespace elixir

using namespace elixir;

extern "C" const char* elixir_last_error(void) { return g_err; }

extern "C" int elixir_ctx_create(elixir_ctx** out, int device, int64_t max_chunk_elems, int max_chunks) {
    if (!out) return fail(ELIXIR_EINVAL, "elixir_ctx_create: out is NULL");
    *out = nullptr;
    if (max_chunk_elems <= 0 || max_chunks <= 0)
        return fail(ELIXIR_EINVAL, "elixir_ctx_create: max_chunk_elems=%lld and max_chunks=%d must be positive",
                    (long long)max_chunk_elems, max_chunks);
    int n_dev = 0;
    ELIXIR_HIP_TRY(hipGetDeviceCount(&n_dev));
    if (device < 0 || device >= n_dev) return fail(ELIXIR_EINVAL, "elixir_ctx_create: device %d of %d", device, n_dev);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(ELIXIR_EHIP, "elixir_ctx_create: cannot make device %d current", device);
    if (const int rc = norm_scratch_init()) return rc;
    elixir_ctx* c = new (std::nothrow) elixir_ctx();
    if (!c) return fail(ELIXIR_EINVAL, "elixir_ctx_create: out of host memory");
    c->device = device;
    c->max_chunk_elems = max_chunk_elems;
    c->max_chunks = max_chunks;
    hipError_t e = hipMalloc((void**)&c->d_partials, sizeof(double) * (size_t)max_chunks * kNormBlocksPerChunk);
    c->stage_len = (max_chunk_elems + 255) / 256 + 1;  // one entry per 256 elements (a wavefront's 4 x 64) + 1 for the odd elements after the last group of 4
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_stage, sizeof(double) * (size_t)c->stage_len);
    if (e != hipSuccess) {
        if (c->d_partials) (void)hipFree(c->d_partials);
        if (c->d_stage) (void)hipFree(c->d_stage);
        delete c;
        return fail(ELIXIR_EHIP, "elixir_ctx_create: %s", hipGetErrorString(e));
    }
    *out = c;
    return ELIXIR_OK;
}

namespace elixir {
void destroy_slots(elixir_ctx* c) {
    for (int i = 0; i < c->n_slots; ++i) {
        if (c->slots[i].ready) (void)hipEventDestroy(c->slots[i].ready);
        if (c->slots[i].updated) (void)hipEventDestroy(c->slots[i].updated);
        if (c->slots[i].evicted) (void)hipEventDestroy(c->slots[i].evicted);
    }
    delete[] c->slots;
    c->slots = nullptr;
    c->n_slots = 0;
    c->slot_bytes = 0;
    c->next_slot = 0;
}
}  // namespace elixir

extern "C" int elixir_ctx_destroy(elixir_ctx* c) {
    if (!c) return ELIXIR_OK;
    DeviceGuard guard(c->device);
    hipError_t e = hipDeviceSynchronize();
    destroy_slots(c);
    if (c->d_partials) (void)hipFree(c->d_partials);
    if (c->d_stage) (void)hipFree(c->d_stage);
    delete c;
    if (e != hipSuccess) return fail(ELIXIR_EHIP, "elixir_ctx_destroy: hipDeviceSynchronize: %s", hipGetErrorString(e));
    return ELIXIR_OK;
}

extern "C" int elixir_host_alloc(void** h_out, size_t bytes) {
    if (!h_out) return fail(ELIXIR_EINVAL, "elixir_host_alloc: h_out is NULL");
    *h_out = nullptr;
    if (bytes == 0) return fail(ELIXIR_EINVAL, "elixir_host_alloc: bytes is 0");
    ELIXIR_HIP_TRY(hipHostMalloc(h_out, bytes, hipHostMallocDefault));
    return ELIXIR_OK;
}

extern "C" int elixir_host_free(void* h_ptr) {
    if (!h_ptr) return ELIXIR_OK;
    ELIXIR_HIP_TRY(hipHostFree(h_ptr));
    return ELIXIR_OK;
}
