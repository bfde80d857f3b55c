// elixir_chunk_adam_step: host side of the fused AdamW update.
#include <math.h>

#include "adam_kernel.hpp"
#include "common.hpp"

using namespace elixir;

namespace {

constexpr int64_t kMaxBlocksPerLaunch = 1ll << 30;  // grid.x stays far below its 2^31 limit; longer chunks take several launches

// Elements [first, first + count) with the vector kernel; count is even and the pointers at `first` are aligned.
template <bool GRAD_BF16, bool HAS_OUT>
void launch_vec(float* p, float* m, float* v, const void* g, uint16_t* out, int64_t first, int64_t count,
                const AdamConsts& c, const float* d_scale, hipStream_t s) {
    const int64_t gsz = GRAD_BF16 ? 2 : 4;
    while (count > 0) {
        const int64_t pairs_all = count / kAdamVec;
        int64_t blocks = (pairs_all + kAdamBlock - 1) / kAdamBlock;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t pairs = pairs_all < blocks * kAdamBlock ? pairs_all : blocks * kAdamBlock;
        hipLaunchKernelGGL((adam_vec_kernel<GRAD_BF16, HAS_OUT>), dim3((unsigned)blocks), dim3(kAdamBlock), kAdamLdsBytes, s,
                           p + first, m + first, v + first, (const void*)((const char*)g + first * gsz),
                           HAS_OUT ? out + first : nullptr, pairs, c, d_scale);
        first += pairs * kAdamVec;
        count -= pairs * kAdamVec;
    }
}

template <bool GRAD_BF16>
void launch_scalar(float* p, float* m, float* v, const void* g, uint16_t* out, int64_t first, int64_t end,
                   const AdamConsts& c, const float* d_scale, hipStream_t s) {
    while (first < end) {
        int64_t blocks = (end - first + 255) / 256;
        if (blocks > kMaxBlocksPerLaunch) blocks = kMaxBlocksPerLaunch;
        const int64_t stop = first + blocks * 256 < end ? first + blocks * 256 : end;
        hipLaunchKernelGGL(adam_scalar_kernel<GRAD_BF16>, dim3((unsigned)blocks), dim3(256), 0, s, p, m, v, g, out, first,
                           stop, c, d_scale);
        first = stop;
    }
}

}  // namespace

extern "C" int elixir_chunk_adam_step(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                                      const uint16_t* d_grad_bf16, uint16_t* d_param_bf16, int64_t n,
                                      const elixir_adam_hparams* hp, const float* d_grad_scale,
                                      elixir_stream_t stream) {
    if (n < 0) return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: n=%lld is negative", (long long)n);
    if (!hp) return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: hp is NULL");
    if (hp->step < 1) return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: step=%lld, steps count from 1", (long long)hp->step);
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: betas must lie in [0, 1)");
    if (!(hp->eps >= 0.0f) || !isfinite(hp->lr) || !isfinite(hp->weight_decay))
        return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: eps must be >= 0 and lr, weight_decay finite");
    if (n == 0) return ELIXIR_OK;
    if ((d_grad_fp32 != nullptr) == (d_grad_bf16 != nullptr))
        return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: exactly one of d_grad_fp32 / d_grad_bf16 must be given");
    if (!d_master || !d_exp_avg || !d_exp_avg_sq)
        return fail(ELIXIR_EINVAL, "elixir_chunk_adam_step: master / exp_avg / exp_avg_sq must not be NULL");
    if (!aligned(d_master, 4) || !aligned(d_exp_avg, 4) || !aligned(d_exp_avg_sq, 4) || !aligned(d_grad_fp32, 4) ||
        !aligned(d_grad_bf16, 2) || !aligned(d_param_bf16, 2) || !aligned(d_grad_scale, 4))
        return fail(ELIXIR_EALIGN, "elixir_chunk_adam_step: a pointer is not aligned for its element type");

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

    hipStream_t s = (hipStream_t)stream;
    const bool bf16 = d_grad_bf16 != nullptr;
    const void* g = bf16 ? (const void*)d_grad_bf16 : (const void*)d_grad_fp32;
    // Vector path: after peeling `head` (0 or 1) elements every fp32 pointer must sit on an 8-byte and every
    // bf16 pointer on a 4-byte boundary.  Whole chunks always do (head = 0).  Anything else, and the odd
    // elements at either end, go to the one-element-per-thread kernel, which computes the same values.
    auto phase = [](const void* q, size_t elem) { return (int)((reinterpret_cast<uintptr_t>(q) / elem) & 1); };
    const int head = phase(d_master, 4);
    const bool vec = phase(d_exp_avg, 4) == head && phase(d_exp_avg_sq, 4) == head && phase(g, bf16 ? 2 : 4) == head &&
                     (!d_param_bf16 || phase(d_param_bf16, 2) == head);
    int64_t vec_first = 0, vec_count = 0;
    if (vec && n - head >= kAdamVec) {
        vec_first = head;
        vec_count = (n - head) / kAdamVec * kAdamVec;
        if (bf16) {
            if (d_param_bf16) launch_vec<true, true>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, vec_first, vec_count, c, d_grad_scale, s);
            else launch_vec<true, false>(d_master, d_exp_avg, d_exp_avg_sq, g, nullptr, vec_first, vec_count, c, d_grad_scale, s);
        } else {
            if (d_param_bf16) launch_vec<false, true>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, vec_first, vec_count, c, d_grad_scale, s);
            else launch_vec<false, false>(d_master, d_exp_avg, d_exp_avg_sq, g, nullptr, vec_first, vec_count, c, d_grad_scale, s);
        }
        ELIXIR_LAUNCH_CHECK("adam_vec_kernel");
    }
    // [0, vec_first) and [vec_first + vec_count, n)
    const int64_t ranges[2][2] = {{0, vec_first}, {vec_first + vec_count, n}};
    for (const auto& r : ranges) {
        if (r[0] >= r[1]) continue;
        if (bf16) launch_scalar<true>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, r[0], r[1], c, d_grad_scale, s);
        else launch_scalar<false>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, r[0], r[1], c, d_grad_scale, s);
        ELIXIR_LAUNCH_CHECK("adam_scalar_kernel");
    }
    return ELIXIR_OK;
}
