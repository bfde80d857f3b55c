// elixir_chunk_adam_step and its variants: host side of the fused AdamW update.
#include <math.h>

#include "adam_kernel.hpp"
#include "common.hpp"
#include "row_plan.hpp"

using namespace elixir;

namespace {

// HIP refuses a launch whose grid spans 2^32 threads or more in x (workgroups here have 128 or 256 threads): longer
// chunks take several launches, and a row of a batched launch is at most kMaxRowBlocks workgroups long
constexpr int64_t kMaxBlocksPerLaunch = ((1ll << 32) - 1) / 256;
constexpr int64_t kMaxRowBlocks = 1ll << 22;

// One request, after validation: element kinds and raw pointers.
struct Req {
    float *p, *m, *v;
    const void* g;
    uint16_t* out;
    int grad_kind;  // kF32 / kBF16 / kF16
    int out_kind;   // kNone / kBF16 / kF16
    const float* d_scale;
    const int32_t* d_skip;
    hipStream_t s;
};

// Calls f.template operator()<GRAD, OUT>() for the run-time (grad_kind, out_kind).
template <typename F>
void dispatch(int grad_kind, int out_kind, F&& f) {
#define ELIXIR_CASE(G, O)                  \
    if (grad_kind == G && out_kind == O) { \
        f.template operator()<G, O>();     \
        return;                            \
    }
    ELIXIR_CASE(kF32, kNone)
    ELIXIR_CASE(kF32, kBF16)
    ELIXIR_CASE(kF32, kF16)
    ELIXIR_CASE(kBF16, kNone)
    ELIXIR_CASE(kBF16, kBF16)
    ELIXIR_CASE(kF16, kNone)
    ELIXIR_CASE(kF16, kF16)
#undef ELIXIR_CASE
}

int64_t grad_elem_size(int grad_kind) { return grad_kind == kF32 ? 4 : 2; }

// Elements [first, first + count) with the vector kernel; count is even and the pointers at `first` are aligned.
struct LaunchVec {
    const Req& r;
    int64_t first, count;
    const AdamConsts& c;
    template <int GRAD, int OUT>
    void operator()() const {
        int64_t at = first, left = count;
        while (left > 0) {
            const int64_t pairs_all = left / kAdamVec;
            int64_t blocks = (pairs_all + kAdamBlock - 1) / kAdamBlock;
            if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
            const int64_t pairs = pairs_all < blocks * kAdamBlock ? pairs_all : blocks * kAdamBlock;
            hipLaunchKernelGGL((adam_vec_kernel<GRAD, OUT>), dim3((unsigned)blocks), dim3(kAdamBlock), kAdamLdsBytes, r.s,
                               r.p + at, r.m + at, r.v + at, (const void*)((const char*)r.g + at * grad_elem_size(GRAD)),
                               OUT != kNone ? r.out + at : nullptr, pairs, r.d_scale, r.d_skip, c);
            at += pairs * kAdamVec;
            left -= pairs * kAdamVec;
        }
    }
};

void launch_scalar(const Req& r, int64_t first, int64_t end, const AdamConsts& c) {
    while (first < end) {
        int64_t blocks = (end - first + 255) / 256;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t stop = first + blocks * 256 < end ? first + blocks * 256 : end;
        const dim3 grid((unsigned)blocks), block(256);
        if (r.grad_kind == kBF16)
            hipLaunchKernelGGL(adam_scalar_kernel<kBF16>, grid, block, 0, r.s, r.p, r.m, r.v, r.g, r.out, r.out_kind, first, stop, c,
                               r.d_scale, r.d_skip);
        else if (r.grad_kind == kF16)
            hipLaunchKernelGGL(adam_scalar_kernel<kF16>, grid, block, 0, r.s, r.p, r.m, r.v, r.g, r.out, r.out_kind, first, stop, c,
                               r.d_scale, r.d_skip);
        else
            hipLaunchKernelGGL(adam_scalar_kernel<kF32>, grid, block, 0, r.s, r.p, r.m, r.v, r.g, r.out, r.out_kind, first, stop, c,
                               r.d_scale, r.d_skip);
        first = stop;
    }
}

int check_hparams(const char* what, const elixir_adam_hparams* hp) {
    if (!hp) return fail(ELIXIR_EINVAL, "%s: hp is NULL", what);
    if (hp->step < 1) return fail(ELIXIR_EINVAL, "%s: step=%lld, steps count from 1", what, (long long)hp->step);
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(ELIXIR_EINVAL, "%s: betas must lie in [0, 1)", what);
    if (!(hp->eps >= 0.0f) || !isfinite(hp->lr) || !isfinite(hp->weight_decay))
        return fail(ELIXIR_EINVAL, "%s: eps must be >= 0 and lr, weight_decay finite", what);
    return ELIXIR_OK;
}

// Step constants in double, rounded once to fp32.
AdamConsts make_consts(const elixir_adam_hparams* hp) {
    const double lr = hp->lr, b1 = hp->beta1, b2 = hp->beta2;
    const double bc1 = 1.0 - pow(b1, (double)hp->step);
    const double bc2 = 1.0 - pow(b2, (double)hp->step);
    AdamConsts c;
    c.lr_wd = (float)(lr * (double)hp->weight_decay);
    c.beta1 = hp->beta1;
    c.omb1 = (float)(1.0 - b1);
    c.beta2 = hp->beta2;
    c.omb2 = (float)(1.0 - b2);
    c.step_size = (float)(lr / bc1);
    c.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
    c.eps = hp->eps;
    return c;
}

// 0 if q sits on a boundary of two elements of size `elem`, 1 if it is one element past such a boundary
int phase(const void* q, size_t elem) { return (int)((reinterpret_cast<uintptr_t>(q) / elem) & 1); }

int lowp_kind(const char* what, int lowp_format, int* kind) {
    if (lowp_format == ELIXIR_LOWP_BF16) *kind = kBF16;
    else if (lowp_format == ELIXIR_LOWP_FP16) *kind = kF16;
    else return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    return ELIXIR_OK;
}

// The single-chunk update after argument checks.
int run_single(const Req& r, int64_t n, const AdamConsts& c) {
    // Vector path: after peeling `head` (0 or 1) elements every fp32 pointer must sit on an 8-byte and every
    // 16-bit pointer on a 4-byte boundary.  Whole chunks always do (head = 0).  Anything else, and the odd
    // elements at either end, go to the one-element-per-thread kernel, which computes the same values.
    const int head = phase(r.p, 4);
    const bool vec = phase(r.m, 4) == head && phase(r.v, 4) == head && phase(r.g, (size_t)grad_elem_size(r.grad_kind)) == head &&
                     (!r.out || phase(r.out, 2) == head);
    int64_t vec_first = 0, vec_count = 0;
    if (vec && n - head >= kAdamVec) {
        vec_first = head;
        vec_count = (n - head) / kAdamVec * kAdamVec;
        dispatch(r.grad_kind, r.out_kind, LaunchVec{r, vec_first, vec_count, c});
        ELIXIR_LAUNCH_CHECK("adam_vec_kernel");
    }
    const int64_t ranges[2][2] = {{0, vec_first}, {vec_first + vec_count, n}};
    for (const auto& rg : ranges) {
        if (rg[0] >= rg[1]) continue;
        launch_scalar(r, rg[0], rg[1], c);
        ELIXIR_LAUNCH_CHECK("adam_scalar_kernel");
    }
    return ELIXIR_OK;
}

}  // namespace

extern "C" int elixir_chunk_adam_step_lp(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                                         const uint16_t* d_grad_lowp, uint16_t* d_param_lowp, int lowp_format, int64_t n,
                                         const elixir_adam_hparams* hp, const float* d_grad_scale, const int32_t* d_skip,
                                         elixir_stream_t stream) {
    static const char* what = "elixir_chunk_adam_step";
    if (n < 0) return fail(ELIXIR_EINVAL, "%s: n=%lld is negative", what, (long long)n);
    if (const int rc = check_hparams(what, hp)) return rc;
    int lk;
    if (const int rc = lowp_kind(what, lowp_format, &lk)) return rc;
    if (n == 0) return ELIXIR_OK;
    if ((d_grad_fp32 != nullptr) == (d_grad_lowp != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of the fp32 and the 16-bit gradient pointer must be given", what);
    if (!d_master || !d_exp_avg || !d_exp_avg_sq)
        return fail(ELIXIR_EINVAL, "%s: master / exp_avg / exp_avg_sq must not be NULL", what);
    if (!aligned(d_master, 4) || !aligned(d_exp_avg, 4) || !aligned(d_exp_avg_sq, 4) || !aligned(d_grad_fp32, 4) ||
        !aligned(d_grad_lowp, 2) || !aligned(d_param_lowp, 2) || !aligned(d_grad_scale, 4) || !aligned(d_skip, 4))
        return fail(ELIXIR_EALIGN, "%s: a pointer is not aligned for its element type", what);
    Req r;
    r.p = d_master;
    r.m = d_exp_avg;
    r.v = d_exp_avg_sq;
    r.g = d_grad_lowp ? (const void*)d_grad_lowp : (const void*)d_grad_fp32;
    r.out = d_param_lowp;
    r.grad_kind = d_grad_lowp ? lk : kF32;
    r.out_kind = d_param_lowp ? lk : kNone;
    r.d_scale = d_grad_scale;
    r.d_skip = d_skip;
    r.s = (hipStream_t)stream;
    return run_single(r, n, make_consts(hp));
}

extern "C" int elixir_chunk_adam_step(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                                      const uint16_t* d_grad_bf16, uint16_t* d_param_bf16, int64_t n,
                                      const elixir_adam_hparams* hp, const float* d_grad_scale,
                                      elixir_stream_t stream) {
    return elixir_chunk_adam_step_lp(d_master, d_exp_avg, d_exp_avg_sq, d_grad_fp32, d_grad_bf16, d_param_bf16,
                                     ELIXIR_LOWP_BF16, n, hp, d_grad_scale, nullptr, stream);
}

// ---- tiled optimizer chunk -------------------------------------------------------------------------------------

namespace {

// d_c: NULL (the constants travel as kernel argument c) or the constants in device memory (c is ignored).
struct LaunchTiled {
    float* state;
    const Req& r;
    int64_t pairs;
    const AdamConsts& c;
    const AdamConsts* d_c;
    template <int GRAD, int OUT>
    void operator()() const {
        const int64_t blocks = (pairs + kAdamBlock - 1) / kAdamBlock;
        if (d_c)
            hipLaunchKernelGGL((adam_tiled_dev_kernel<GRAD, OUT>), dim3((unsigned)blocks), dim3(kAdamBlock), kAdamLdsBytes, r.s, state, r.g,
                               OUT != kNone ? r.out : nullptr, pairs, d_c, r.d_scale, r.d_skip);
        else
            hipLaunchKernelGGL((adam_tiled_kernel<GRAD, OUT>), dim3((unsigned)blocks), dim3(kAdamBlock), kAdamLdsBytes, r.s, state, r.g,
                               OUT != kNone ? r.out : nullptr, pairs, r.d_scale, r.d_skip, c);
    }
};

void launch_tiled_scalar(float* state, const Req& r, int64_t first, int64_t end, const AdamConsts& c, const AdamConsts* d_c = nullptr) {
    while (first < end) {
        int64_t blocks = (end - first + 255) / 256;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t stop = first + blocks * 256 < end ? first + blocks * 256 : end;
        const dim3 grid((unsigned)blocks), block(256);
        if (r.grad_kind == kBF16)
            hipLaunchKernelGGL(adam_tiled_scalar_kernel<kBF16>, grid, block, 0, r.s, state, r.g, r.out, r.out_kind, first, stop, c, d_c, r.d_scale, r.d_skip);
        else if (r.grad_kind == kF16)
            hipLaunchKernelGGL(adam_tiled_scalar_kernel<kF16>, grid, block, 0, r.s, state, r.g, r.out, r.out_kind, first, stop, c, d_c, r.d_scale, r.d_skip);
        else
            hipLaunchKernelGGL(adam_tiled_scalar_kernel<kF32>, grid, block, 0, r.s, state, r.g, r.out, r.out_kind, first, stop, c, d_c, r.d_scale, r.d_skip);
        first = stop;
    }
}

}  // namespace

extern "C" int64_t elixir_state_tiled_len(int64_t n) {
    return n <= 0 ? 0 : 3 * kStateTile * ((n + kStateTile - 1) / kStateTile);
}

namespace {
// hp (constants derived on the host, travelling as kernel argument) or d_st (constants in device memory): exactly one.
int tiled_step(const char* what, float* d_state, const float* d_grad_fp32, const uint16_t* d_grad_lowp, uint16_t* d_param_lowp,
               int lowp_format, int64_t n, const elixir_adam_hparams* hp, const elixir_adam_step_state* d_st,
               const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream) {
    if (n < 0) return fail(ELIXIR_EINVAL, "%s: n=%lld is negative", what, (long long)n);
    if (!d_st) {
        if (const int rc = check_hparams(what, hp)) return rc;
    } else if (!aligned(d_st, 8)) {
        return fail(ELIXIR_EALIGN, "%s: the step state must be 8-byte aligned", what);
    }
    int lk;
    if (const int rc = lowp_kind(what, lowp_format, &lk)) return rc;
    if (n == 0) return ELIXIR_OK;
    if ((d_grad_fp32 != nullptr) == (d_grad_lowp != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of the fp32 and the 16-bit gradient pointer must be given", what);
    if (!d_state) return fail(ELIXIR_EINVAL, "%s: d_state is NULL", what);
    if (!aligned(d_state, 8) || !aligned(d_grad_fp32, 4) || !aligned(d_grad_lowp, 2) || !aligned(d_param_lowp, 2) ||
        !aligned(d_grad_scale, 4) || !aligned(d_skip, 4))
        return fail(ELIXIR_EALIGN, "%s: d_state must be 8-byte aligned, the other pointers aligned for their element type", what);
    if (n / kAdamVec / kAdamBlock >= kMaxBlocksPerLaunch)
        return fail(ELIXIR_ECAP, "%s: a chunk of %lld elements does not fit one launch", what, (long long)n);
    Req r;
    r.p = r.m = r.v = nullptr;
    r.g = d_grad_lowp ? (const void*)d_grad_lowp : (const void*)d_grad_fp32;
    r.out = d_param_lowp;
    r.grad_kind = d_grad_lowp ? lk : kF32;
    r.out_kind = d_param_lowp ? lk : kNone;
    r.d_scale = d_grad_scale;
    r.d_skip = d_skip;
    r.s = (hipStream_t)stream;
    const AdamConsts c = d_st ? AdamConsts{} : make_consts(hp);
    const AdamConsts* d_c = d_st ? reinterpret_cast<const AdamConsts*>(d_st->consts) : nullptr;   // an address, not a read: d_st is device memory
    // the vector kernel wants the gradient on an 8-byte (fp32) or 4-byte (16-bit) boundary and the copy on a 4-byte one;
    // whole chunks are; anything else, and an odd last element, takes the one-element kernel
    const bool vec = phase(r.g, (size_t)grad_elem_size(r.grad_kind)) == 0 && (!r.out || phase(r.out, 2) == 0) && n >= kAdamVec;
    int64_t done = 0;
    if (vec) {
        dispatch(r.grad_kind, r.out_kind, LaunchTiled{d_state, r, n / kAdamVec, c, d_c});
        ELIXIR_LAUNCH_CHECK("adam_tiled_kernel");
        done = n / kAdamVec * kAdamVec;
    }
    if (done < n) {
        launch_tiled_scalar(d_state, r, done, n, c, d_c);
        ELIXIR_LAUNCH_CHECK("adam_tiled_scalar_kernel");
    }
    return ELIXIR_OK;
}
}  // namespace

extern "C" int elixir_chunk_adam_step_tiled_lp(float* d_state, const float* d_grad_fp32, const uint16_t* d_grad_lowp,
                                               uint16_t* d_param_lowp, int lowp_format, int64_t n,
                                               const elixir_adam_hparams* hp, const float* d_grad_scale,
                                               const int32_t* d_skip, elixir_stream_t stream) {
    return tiled_step("elixir_chunk_adam_step_tiled", d_state, d_grad_fp32, d_grad_lowp, d_param_lowp, lowp_format, n, hp, nullptr,
                      d_grad_scale, d_skip, stream);
}

extern "C" int elixir_chunk_adam_step_tiled_dev(float* d_state, const float* d_grad_fp32, const uint16_t* d_grad_lowp,
                                                uint16_t* d_param_lowp, int lowp_format, int64_t n,
                                                const elixir_adam_step_state* d_step_state, const float* d_grad_scale,
                                                const int32_t* d_skip, elixir_stream_t stream) {
    static const char* what = "elixir_chunk_adam_step_tiled_dev";
    if (!d_step_state) return fail(ELIXIR_EINVAL, "%s: d_step_state is NULL", what);
    return tiled_step(what, d_state, d_grad_fp32, d_grad_lowp, d_param_lowp, lowp_format, n, nullptr, d_step_state, d_grad_scale,
                      d_skip, stream);
}

namespace {

// flat <-> tiled: one element per thread, blockIdx.y = which of the three arrays
template <bool TO_TILED>
__global__ __launch_bounds__(256) void state_tile_kernel(float* tiled, float* a0, float* a1, float* a2, int64_t n, int64_t padded) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= padded) return;
    float* arr = blockIdx.y == 0 ? a0 : (blockIdx.y == 1 ? a1 : a2);
    float* T = tiled + 3 * kStateTile * (e / kStateTile) + (int64_t)blockIdx.y * kStateTile + e % kStateTile;
    if constexpr (TO_TILED) *T = e < n ? arr[e] : 0.0f;
    else if (e < n) arr[e] = *T;
}

// The same with one 128-bit access per lane in single-wavefront workgroups (all four pointers 16-byte aligned): group
// g holds elements 4g .. 4g+3, which lie in one tile (a tile is a multiple of 4 elements); the group that straddles n
// goes element by element.
typedef float tile_f32x4 __attribute__((ext_vector_type(4)));

template <bool TO_TILED>
__global__ __launch_bounds__(64) void state_tile_vec_kernel(float* tiled, float* a0, float* a1, float* a2, int64_t n, int64_t padded) {
    const int64_t e = ((int64_t)blockIdx.x * 64 + threadIdx.x) * 4;
    if (e >= padded) return;
    float* arr = blockIdx.y == 0 ? a0 : (blockIdx.y == 1 ? a1 : a2);
    float* T = tiled + 3 * kStateTile * (e / kStateTile) + (int64_t)blockIdx.y * kStateTile + e % kStateTile;
    if (e + 4 <= n) {
        if constexpr (TO_TILED) __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const tile_f32x4*>(arr + e)), reinterpret_cast<tile_f32x4*>(T));
        else __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const tile_f32x4*>(T)), reinterpret_cast<tile_f32x4*>(arr + e));
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (TO_TILED) T[j] = e + j < n ? arr[e + j] : 0.0f;
        else if (e + j < n) arr[e + j] = T[j];
    }
}

template <bool TO_TILED>
int tile_call(const char* what, float* tiled, float* a0, float* a1, float* a2, int64_t n, hipStream_t s) {
    if (n < 0) return fail(ELIXIR_EINVAL, "%s: n is negative", what);
    if (n == 0) return ELIXIR_OK;
    if (!tiled || !a0 || !a1 || !a2) return fail(ELIXIR_EINVAL, "%s: NULL pointer", what);
    if (!aligned(tiled, 4) || !aligned(a0, 4) || !aligned(a1, 4) || !aligned(a2, 4)) return fail(ELIXIR_EALIGN, "%s: pointer not 4-byte aligned", what);
    const int64_t padded = (n + kStateTile - 1) / kStateTile * kStateTile;
    if (padded / 256 >= kMaxBlocksPerLaunch) return fail(ELIXIR_ECAP, "%s: %lld elements do not fit one launch", what, (long long)n);
    if (aligned(tiled, 16) && aligned(a0, 16) && aligned(a1, 16) && aligned(a2, 16))
        hipLaunchKernelGGL((state_tile_vec_kernel<TO_TILED>), dim3((unsigned)(padded / 256), 3), dim3(64), 0, s, tiled, a0, a1, a2, n, padded);
    else
        hipLaunchKernelGGL((state_tile_kernel<TO_TILED>), dim3((unsigned)(padded / 256), 3), dim3(256), 0, s, tiled, a0, a1, a2, n, padded);
    ELIXIR_LAUNCH_CHECK("state_tile_kernel");
    return ELIXIR_OK;
}

}  // namespace

extern "C" int elixir_state_tile(float* d_state, const float* d_master, const float* d_exp_avg, const float* d_exp_avg_sq, int64_t n,
                                 elixir_stream_t stream) {
    return tile_call<true>("elixir_state_tile", d_state, const_cast<float*>(d_master), const_cast<float*>(d_exp_avg),
                           const_cast<float*>(d_exp_avg_sq), n, (hipStream_t)stream);
}

extern "C" int elixir_state_untile(const float* d_state, float* d_master, float* d_exp_avg, float* d_exp_avg_sq, int64_t n,
                                   elixir_stream_t stream) {
    return tile_call<false>("elixir_state_untile", const_cast<float*>(d_state), d_master, d_exp_avg, d_exp_avg_sq, n, (hipStream_t)stream);
}

namespace {

struct LaunchMulti {
    const AdamMultiTable& tab;
    dim3 grid;
    const AdamConsts& c;
    const AdamConsts* d_c;  // tiled only: the constants in device memory, taken instead of c
    const float* d_scale;
    const int32_t* d_skip;
    hipStream_t s;
    bool tiled;
    template <int GRAD, int OUT>
    void operator()() const {
        if (tiled && d_c) hipLaunchKernelGGL((adam_multi_dev_kernel<GRAD, OUT>), grid, dim3(kAdamBlock), kAdamLdsBytes, s, tab, d_c, d_scale, d_skip);
        else if (tiled) hipLaunchKernelGGL((adam_multi_kernel<GRAD, OUT, true>), grid, dim3(kAdamBlock), kAdamLdsBytes, s, tab, c, d_scale, d_skip);
        else hipLaunchKernelGGL((adam_multi_kernel<GRAD, OUT, false>), grid, dim3(kAdamBlock), kAdamLdsBytes, s, tab, c, d_scale, d_skip);
    }
};

// The batched update.  tiled: d_master[k] is the tiled optimizer chunk of chunk k and the two moment tables are unused.
int adam_multi(const char* what, bool tiled, int n_chunks, float* const* d_master, float* const* d_exp_avg,
               float* const* d_exp_avg_sq, const float* const* d_grad_fp32, const uint16_t* const* d_grad_lowp,
               uint16_t* const* d_param_lowp, int lowp_format, const int64_t* n, const elixir_adam_hparams* hp,
               const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream,
               const elixir_adam_step_state* d_st = nullptr) {  // d_st (tiled only): constants from device memory, hp unused
    if (n_chunks < 0) return fail(ELIXIR_EINVAL, "%s: n_chunks is negative", what);
    if (!d_st) {
        if (const int rc = check_hparams(what, hp)) return rc;
    } else if (!aligned(d_st, 8)) {
        return fail(ELIXIR_EALIGN, "%s: the step state must be 8-byte aligned", what);
    }
    int lk;
    if (const int rc = lowp_kind(what, lowp_format, &lk)) return rc;
    if (n_chunks == 0) return ELIXIR_OK;
    if (!d_master || (!tiled && (!d_exp_avg || !d_exp_avg_sq)) || !n) return fail(ELIXIR_EINVAL, "%s: NULL table", what);
    if ((d_grad_fp32 != nullptr) == (d_grad_lowp != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of the fp32 and the 16-bit gradient table must be given", what);
    if (!aligned(d_grad_scale, 4) || !aligned(d_skip, 4)) return fail(ELIXIR_EALIGN, "%s: d_grad_scale / d_skip not 4-byte aligned", what);
    const bool lowp_grad = d_grad_lowp != nullptr;
    const int grad_kind = lowp_grad ? lk : kF32;
    const int out_kind = d_param_lowp ? lk : kNone;
    const size_t gsz = (size_t)grad_elem_size(grad_kind);
    for (int k = 0; k < n_chunks; ++k) {
        if (n[k] < 0) return fail(ELIXIR_EINVAL, "%s: n[%d] is negative", what, k);
        if (n[k] == 0) continue;
        const void* g = lowp_grad ? (const void*)d_grad_lowp[k] : (const void*)d_grad_fp32[k];
        if (!d_master[k] || (!tiled && (!d_exp_avg[k] || !d_exp_avg_sq[k])) || !g) return fail(ELIXIR_EINVAL, "%s: NULL pointer in chunk %d", what, k);
        if (!aligned(d_master[k], tiled ? 8 : 4) || (!tiled && (!aligned(d_exp_avg[k], 4) || !aligned(d_exp_avg_sq[k], 4))) || !aligned(g, gsz) ||
            (d_param_lowp && !aligned(d_param_lowp[k], 2)))
            return fail(ELIXIR_EALIGN, "%s: a pointer of chunk %d is not aligned for its element type%s", what, k,
                        tiled ? " (8 bytes for a tiled optimizer chunk)" : "");
        if (d_param_lowp && !d_param_lowp[k]) return fail(ELIXIR_EINVAL, "%s: the parameter-copy pointer of chunk %d is NULL", what, k);
    }
    const AdamConsts c = d_st ? AdamConsts{} : make_consts(hp);
    const AdamConsts* d_c = d_st ? reinterpret_cast<const AdamConsts*>(d_st->consts) : nullptr;  // an address, not a read
    hipStream_t s = (hipStream_t)stream;
    AdamMultiTable tab;
    int in_table = 0;
    int64_t max_blocks = 0;  // grid row length
    auto flush = [&]() -> int {
        if (in_table == 0) return ELIXIR_OK;
        for (int j = in_table; j < kAdamMultiMax; ++j) {
            tab.master[j] = tab.exp_avg[j] = tab.exp_avg_sq[j] = nullptr;
            tab.grad[j] = nullptr;
            tab.out[j] = nullptr;
            tab.n2[j] = 0;
        }
        dispatch(grad_kind, out_kind, LaunchMulti{tab, dim3((unsigned)max_blocks, (unsigned)in_table), c, d_c, d_grad_scale, d_skip, s, tiled});
        ELIXIR_LAUNCH_CHECK("adam_multi_kernel");
        in_table = 0;
        max_blocks = 0;
        return ELIXIR_OK;
    };
    auto make_req = [&](int k) {
        Req r;
        r.p = d_master[k];
        r.m = tiled ? nullptr : d_exp_avg[k];
        r.v = tiled ? nullptr : d_exp_avg_sq[k];
        r.g = lowp_grad ? (const void*)d_grad_lowp[k] : (const void*)d_grad_fp32[k];
        r.out = d_param_lowp ? d_param_lowp[k] : nullptr;
        r.grad_kind = grad_kind;
        r.out_kind = out_kind;
        r.d_scale = d_grad_scale;
        r.d_skip = d_skip;
        r.s = s;
        return r;
    };
    // chunks that qualify for the vector kernel go through the row plan (row_plan.hpp): grid rows are equal pieces of
    // the chunks plus a tail each, tails of similar length share a launch.  With a handful of ragged chunks whole
    // chunks as rows leave a third of the workgroups without work (seven 4Mi-element chunks of a 21M-parameter set:
    // 80.6% of the HBM peak, 82.3% with pieces); with hundreds of chunks the rows are the chunks, grouped by length
    // (the 251 8Mi-element chunks of the 1.5B set: 86.1%).  A piece is a whole number of state tiles, so its base
    // pointers are those of the chunk shifted.
    constexpr int64_t kTileBlocks = kStateTile / (kAdamBlock * kAdamVec);
    auto vec_ok = [&](int k) {
        if (n[k] < kAdamVec) return false;
        const Req r = make_req(k);
        return (tiled || (phase(r.p, 4) == 0 && phase(r.m, 4) == 0 && phase(r.v, 4) == 0)) && phase(r.g, gsz) == 0 &&
               (!r.out || phase(r.out, 2) == 0);
    };
    for (int k = 0; k < n_chunks; ++k) {
        if (n[k] == 0) continue;
        const Req r = make_req(k);
        if (!vec_ok(k)) {  // a slice at an odd offset: the single-chunk path
            if (tiled) {
                launch_tiled_scalar(r.p, r, 0, n[k], c, d_c);
                ELIXIR_LAUNCH_CHECK("adam_tiled_scalar_kernel");
            } else if (const int rc = run_single(r, n[k], c)) {
                return rc;
            }
        } else if (n[k] % kAdamVec) {  // the odd last element of this chunk
            const int64_t done = n[k] / kAdamVec * kAdamVec;
            if (tiled) launch_tiled_scalar(r.p, r, done, n[k], c, d_c);
            else launch_scalar(r, done, n[k], c);
            ELIXIR_LAUNCH_CHECK("adam_scalar_kernel");
        }
    }
    struct Rows {
        decltype(make_req)& req;
        decltype(flush)& flush_table;
        AdamMultiTable& tab;
        int& in_table;
        int64_t& max_blocks;
        const int64_t* n;
        bool tiled;
        size_t gsz;
        void add(int k, int64_t first_block, int64_t n_blocks) {
            const Req r = req(k);
            const int64_t e0 = first_block * kAdamBlock * kAdamVec;  // first element of the piece: a multiple of the state tile
            int64_t pairs = n[k] / kAdamVec - first_block * kAdamBlock;
            if (pairs > n_blocks * kAdamBlock) pairs = n_blocks * kAdamBlock;
            const int j = in_table++;
            tab.master[j] = tiled ? r.p + 3 * e0 : r.p + e0;
            tab.exp_avg[j] = tiled ? nullptr : r.m + e0;
            tab.exp_avg_sq[j] = tiled ? nullptr : r.v + e0;
            tab.grad[j] = (const char*)r.g + e0 * (int64_t)gsz;
            tab.out[j] = r.out ? r.out + e0 : nullptr;
            tab.n2[j] = pairs;
        }
        int flush(int64_t row_blocks) {
            max_blocks = row_blocks;
            return flush_table();
        }
    } rows{make_req, flush, tab, in_table, max_blocks, n, tiled, gsz};
    auto blocks_of = [&](int k) -> int64_t { return vec_ok(k) ? (n[k] / kAdamVec + kAdamBlock - 1) / kAdamBlock : 0; };
    return plan_rows(n_chunks, blocks_of, kTileBlocks, kAdamMultiMax, kMaxRowBlocks / kTileBlocks * kTileBlocks, rows);
}

}  // namespace

extern "C" int elixir_chunk_adam_step_multi_lp(int n_chunks, float* const* d_master, float* const* d_exp_avg,
                                               float* const* d_exp_avg_sq, const float* const* d_grad_fp32,
                                               const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp,
                                               int lowp_format, const int64_t* n, const elixir_adam_hparams* hp,
                                               const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream) {
    return no_throw("elixir_chunk_adam_step_multi", [&] {
        return adam_multi("elixir_chunk_adam_step_multi", false, n_chunks, d_master, d_exp_avg, d_exp_avg_sq, d_grad_fp32, d_grad_lowp,
                          d_param_lowp, lowp_format, n, hp, d_grad_scale, d_skip, stream);
    });
}

extern "C" int elixir_chunk_adam_step_tiled_multi_lp(int n_chunks, float* const* d_state, const float* const* d_grad_fp32,
                                                     const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp,
                                                     int lowp_format, const int64_t* n, const elixir_adam_hparams* hp,
                                                     const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream) {
    return no_throw("elixir_chunk_adam_step_tiled_multi", [&] {
        return adam_multi("elixir_chunk_adam_step_tiled_multi", true, n_chunks, d_state, nullptr, nullptr, d_grad_fp32, d_grad_lowp,
                          d_param_lowp, lowp_format, n, hp, d_grad_scale, d_skip, stream);
    });
}

extern "C" int elixir_chunk_adam_step_tiled_multi_dev(int n_chunks, float* const* d_state, const float* const* d_grad_fp32,
                                                      const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp,
                                                      int lowp_format, const int64_t* n, const elixir_adam_step_state* d_step_state,
                                                      const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream) {
    if (!d_step_state) return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step_tiled_multi_dev: d_step_state is NULL");
    return no_throw("elixir_chunk_adam_step_tiled_multi_dev", [&] {
        return adam_multi("elixir_chunk_adam_step_tiled_multi_dev", true, n_chunks, d_state, nullptr, nullptr, d_grad_fp32, d_grad_lowp,
                          d_param_lowp, lowp_format, n, nullptr, d_grad_scale, d_skip, stream, d_step_state);
    });
}

// ---- the step state in device memory ---------------------------------------------------------------------------
//
// A launch whose constants are kernel arguments belongs to one step number; a captured graph of such launches
// replays that step number for ever.  The step state keeps the hyper-parameters, the count of steps done and the
// constants of the current step in device memory: elixir_adam_step_state_advance (one thread) counts one step on and
// derives the constants exactly as make_consts does on the host (double precision, rounded once to fp32), unless the
// step is being skipped; the *_dev updates read them from there.  Captured together, advance + updates replay as
// steps t, t+1, t+2, ...

namespace {

__global__ void adam_state_init_kernel(elixir_adam_step_state* st, elixir_adam_hparams hp) {
    st->lr = hp.lr;
    st->beta1 = hp.beta1;
    st->beta2 = hp.beta2;
    st->eps = hp.eps;
    st->weight_decay = hp.weight_decay;
    st->reserved = 0;
    st->step = hp.step - 1;  // steps done: the first advance makes hp.step the current step
    for (int k = 0; k < 8; ++k) st->consts[k] = 0.0f;
}

__global__ void adam_state_advance_kernel(elixir_adam_step_state* st, const int32_t* d_skip) {
    if (d_skip && *d_skip) return;  // a skipped step does not count
    const int64_t t = st->step + 1;
    st->step = t;
    const double lr = st->lr, b1 = st->beta1, b2 = st->beta2;
    const double bc1 = 1.0 - pow(b1, (double)t);
    const double bc2 = 1.0 - pow(b2, (double)t);
    AdamConsts c;
    c.lr_wd = (float)(lr * (double)st->weight_decay);
    c.beta1 = st->beta1;
    c.omb1 = (float)(1.0 - b1);
    c.beta2 = st->beta2;
    c.omb2 = (float)(1.0 - b2);
    c.step_size = (float)(lr / bc1);
    c.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
    c.eps = st->eps;
    *reinterpret_cast<AdamConsts*>(st->consts) = c;
}

}  // namespace

extern "C" int elixir_adam_step_state_init(elixir_adam_step_state* d_step_state, const elixir_adam_hparams* hp, elixir_stream_t stream) {
    static const char* what = "elixir_adam_step_state_init";
    if (!d_step_state) return fail(ELIXIR_EINVAL, "%s: d_step_state is NULL", what);
    if (!aligned(d_step_state, 8)) return fail(ELIXIR_EALIGN, "%s: d_step_state must be 8-byte aligned", what);
    if (const int rc = check_hparams(what, hp)) return rc;
    hipLaunchKernelGGL(adam_state_init_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, d_step_state, *hp);
    ELIXIR_LAUNCH_CHECK("adam_state_init_kernel");
    return ELIXIR_OK;
}

extern "C" int elixir_adam_step_state_advance(elixir_adam_step_state* d_step_state, const int32_t* d_skip, elixir_stream_t stream) {
    static const char* what = "elixir_adam_step_state_advance";
    if (!d_step_state) return fail(ELIXIR_EINVAL, "%s: d_step_state is NULL", what);
    if (!aligned(d_step_state, 8) || !aligned(d_skip, 4)) return fail(ELIXIR_EALIGN, "%s: pointer not aligned", what);
    hipLaunchKernelGGL(adam_state_advance_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, d_step_state, d_skip);
    ELIXIR_LAUNCH_CHECK("adam_state_advance_kernel");
    return ELIXIR_OK;
}

extern "C" int elixir_chunk_adam_step_multi(int n_chunks, float* const* d_master, float* const* d_exp_avg,
                                            float* const* d_exp_avg_sq, const float* const* d_grad_fp32,
                                            const uint16_t* const* d_grad_bf16, uint16_t* const* d_param_bf16,
                                            const int64_t* n, const elixir_adam_hparams* hp, const float* d_grad_scale,
                                            elixir_stream_t stream) {
    return elixir_chunk_adam_step_multi_lp(n_chunks, d_master, d_exp_avg, d_exp_avg_sq, d_grad_fp32, d_grad_bf16, d_param_bf16,
                                           ELIXIR_LOWP_BF16, n, hp, d_grad_scale, nullptr, stream);
}

// ---- dynamic loss scaling (fp16 gradients) -------------------------------------------------------------------
//
// Loss scaling as in Micikevicius et al., "Mixed Precision Training" (the reference the paper gives for its fp16
// set-up): the loss is multiplied by S so that small gradients survive fp16; an Inf/NaN among the gradients means
// S was too large -- the step is skipped and S shrinks; after growth_interval clean steps S grows.  The state
// lives in device memory and is advanced by a one-thread kernel from the norm that elixir_chunk_grad_norm left
// there (a non-finite norm is the overflow signal: the fp64 sum of finite fp32 squares cannot overflow), so the
// host never waits.

namespace {

__global__ void loss_scale_init_kernel(elixir_loss_scale_state* st, float init_scale) {
    st->scale = init_scale;
    st->good_steps = 0;
    st->skip = 0;
    st->grad_scale = 1.0f / init_scale;
}

__global__ void loss_scale_update_kernel(elixir_loss_scale_state* st, const float* d_norm_scaled, float max_norm,
                                         float growth_factor, float backoff_factor, int growth_interval) {
    const float norm = *d_norm_scaled;
    const float S = st->scale;
    if (!(fabsf(norm) <= 3.402823466e38f)) {  // Inf or NaN
        st->scale = S * backoff_factor;
        st->good_steps = 0;
        st->skip = 1;
        st->grad_scale = 0.0f;
        return;
    }
    double coef = 1.0;
    if (max_norm > 0.0f) {
        const double r = (double)max_norm / ((double)norm / (double)S + 1e-6);
        coef = r < 1.0 ? r : 1.0;
    }
    st->grad_scale = (float)(coef / (double)S);
    st->skip = 0;
    int good = st->good_steps + 1;
    if (good >= growth_interval) {
        st->scale = S * growth_factor;
        good = 0;
    }
    st->good_steps = good;
}

}  // namespace

extern "C" int elixir_loss_scale_init(elixir_loss_scale_state* d_state, float init_scale, elixir_stream_t stream) {
    if (!d_state || !aligned(d_state, 4)) return fail(d_state ? ELIXIR_EALIGN : ELIXIR_EINVAL, "elixir_loss_scale_init: bad d_state");
    if (!(init_scale > 0.0f) || !isfinite(init_scale))
        return fail(ELIXIR_EINVAL, "elixir_loss_scale_init: init_scale must be positive and finite");
    hipLaunchKernelGGL(loss_scale_init_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, d_state, init_scale);
    ELIXIR_LAUNCH_CHECK("loss_scale_init_kernel");
    return ELIXIR_OK;
}

extern "C" int elixir_loss_scale_update(elixir_loss_scale_state* d_state, const float* d_norm_scaled, float max_norm,
                                        float growth_factor, float backoff_factor, int growth_interval,
                                        elixir_stream_t stream) {
    static const char* what = "elixir_loss_scale_update";
    if (!d_state || !d_norm_scaled) return fail(ELIXIR_EINVAL, "%s: NULL pointer", what);
    if (!aligned(d_state, 4) || !aligned(d_norm_scaled, 4)) return fail(ELIXIR_EALIGN, "%s: pointer not 4-byte aligned", what);
    if (!(growth_factor >= 1.0f) || !(backoff_factor > 0.0f && backoff_factor <= 1.0f) || growth_interval < 1)
        return fail(ELIXIR_EINVAL, "%s: need growth_factor >= 1, 0 < backoff_factor <= 1, growth_interval >= 1", what);
    hipLaunchKernelGGL(loss_scale_update_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, d_state, d_norm_scaled, max_norm,
                       growth_factor, backoff_factor, growth_interval);
    ELIXIR_LAUNCH_CHECK("loss_scale_update_kernel");
    return ELIXIR_OK;
}
