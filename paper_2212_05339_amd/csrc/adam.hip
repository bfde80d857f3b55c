// elixir_chunk_adam_step: host side of the fused AdamW update.
#include <math.h>

#include "adam_kernel.hpp"
#include "common.hpp"

using namespace elixir;

namespace {

// Launch shape of the vector kernel (chosen by measurement on MI355X).
constexpr int kUnroll = 4;
constexpr bool kNtLoad = true;
constexpr bool kNtStore = true;
constexpr int64_t kMaxGrid = 256 * 16;  // workgroups: 16 per compute unit, grid-stride beyond that

template <bool GRAD_BF16, bool HAS_OUT>
void launch_vec(float* p, float* m, float* v, const void* g, uint16_t* out, int64_t n4, const AdamConsts& c,
                const float* d_scale, hipStream_t s) {
    const int64_t tiles = (n4 + 256 * kUnroll - 1) / (256 * kUnroll);
    const unsigned grid = (unsigned)(tiles < kMaxGrid ? tiles : kMaxGrid);
    hipLaunchKernelGGL((adam_vec_kernel<GRAD_BF16, HAS_OUT, kUnroll, kNtLoad, kNtStore>), dim3(grid), dim3(256), 0, s,
                       p, m, v, g, out, n4, c, d_scale);
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
    c.decay = (float)(1.0 - lr * (double)hp->weight_decay);
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
    const bool vec = aligned(d_master, 16) && aligned(d_exp_avg, 16) && aligned(d_exp_avg_sq, 16) &&
                     aligned(g, bf16 ? 8 : 16) && aligned(d_param_bf16, 8);
    int64_t done = 0;
    if (vec && n >= 4) {
        const int64_t n4 = n / 4;
        if (bf16) {
            if (d_param_bf16) launch_vec<true, true>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, n4, c, d_grad_scale, s);
            else launch_vec<true, false>(d_master, d_exp_avg, d_exp_avg_sq, g, nullptr, n4, c, d_grad_scale, s);
        } else {
            if (d_param_bf16) launch_vec<false, true>(d_master, d_exp_avg, d_exp_avg_sq, g, d_param_bf16, n4, c, d_grad_scale, s);
            else launch_vec<false, false>(d_master, d_exp_avg, d_exp_avg_sq, g, nullptr, n4, c, d_grad_scale, s);
        }
        ELIXIR_LAUNCH_CHECK("adam_vec_kernel");
        done = n4 * 4;
    }
    if (done < n) {  // misaligned buffers, or the last n % 4 elements
        const int64_t rest = n - done;
        int64_t blocks = (rest + 255) / 256;
        if (blocks > 256 * 8) blocks = 256 * 8;
        if (bf16) hipLaunchKernelGGL(adam_scalar_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, d_master, d_exp_avg,
                                     d_exp_avg_sq, g, d_param_bf16, done, n, c, d_grad_scale);
        else hipLaunchKernelGGL(adam_scalar_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, d_master, d_exp_avg,
                                d_exp_avg_sq, g, d_param_bf16, done, n, c, d_grad_scale);
        ELIXIR_LAUNCH_CHECK("adam_scalar_kernel");
    }
    return ELIXIR_OK;
}
