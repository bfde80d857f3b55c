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

}  // namespace

extern "C" int elixir_chunk_adam_step(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                                      const uint16_t* d_grad_bf16, uint16_t* d_param_bf16, int64_t n,
                                      const elixir_adam_hparams* hp, const float* d_grad_scale,
                                      elixir_stream_t stream) {
    static const char* what = "elixir_chunk_adam_step";
    if (n < 0) return fail(ELIXIR_EINVAL, "%s: n=%lld is negative", what, (long long)n);
    if (const int rc = check_hparams(what, hp)) return rc;
    if (n == 0) return ELIXIR_OK;
    if ((d_grad_fp32 != nullptr) == (d_grad_bf16 != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of d_grad_fp32 / d_grad_bf16 must be given", what);
    if (!d_master || !d_exp_avg || !d_exp_avg_sq)
        return fail(ELIXIR_EINVAL, "%s: master / exp_avg / exp_avg_sq must not be NULL", what);
    if (!aligned(d_master, 4) || !aligned(d_exp_avg, 4) || !aligned(d_exp_avg_sq, 4) || !aligned(d_grad_fp32, 4) ||
        !aligned(d_grad_bf16, 2) || !aligned(d_param_bf16, 2) || !aligned(d_grad_scale, 4))
        return fail(ELIXIR_EALIGN, "%s: a pointer is not aligned for its element type", what);
    const AdamConsts c = make_consts(hp);

    hipStream_t s = (hipStream_t)stream;
    const bool bf16 = d_grad_bf16 != nullptr;
    const void* g = bf16 ? (const void*)d_grad_bf16 : (const void*)d_grad_fp32;
    // Vector path: after peeling `head` (0 or 1) elements every fp32 pointer must sit on an 8-byte and every
    // bf16 pointer on a 4-byte boundary.  Whole chunks always do (head = 0).  Anything else, and the odd
    // elements at either end, go to the one-element-per-thread kernel, which computes the same values.
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

extern "C" int elixir_chunk_adam_step_multi(int n_chunks, float* const* d_master, float* const* d_exp_avg,
                                            float* const* d_exp_avg_sq, const float* const* d_grad_fp32,
                                            const uint16_t* const* d_grad_bf16, uint16_t* const* d_param_bf16,
                                            const int64_t* n, const elixir_adam_hparams* hp, const float* d_grad_scale,
                                            elixir_stream_t stream) {
    static const char* what = "elixir_chunk_adam_step_multi";
    if (n_chunks < 0) return fail(ELIXIR_EINVAL, "%s: n_chunks is negative", what);
    if (const int rc = check_hparams(what, hp)) return rc;
    if (n_chunks == 0) return ELIXIR_OK;
    if (!d_master || !d_exp_avg || !d_exp_avg_sq || !n) return fail(ELIXIR_EINVAL, "%s: NULL table", what);
    if ((d_grad_fp32 != nullptr) == (d_grad_bf16 != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of d_grad_fp32 / d_grad_bf16 must be given", what);
    if (!aligned(d_grad_scale, 4)) return fail(ELIXIR_EALIGN, "%s: d_grad_scale not 4-byte aligned", what);
    const bool bf16 = d_grad_bf16 != nullptr;
    for (int k = 0; k < n_chunks; ++k) {
        if (n[k] < 0) return fail(ELIXIR_EINVAL, "%s: n[%d] is negative", what, k);
        if (n[k] == 0) continue;
        const void* g = bf16 ? (const void*)d_grad_bf16[k] : (const void*)d_grad_fp32[k];
        if (!d_master[k] || !d_exp_avg[k] || !d_exp_avg_sq[k] || !g) return fail(ELIXIR_EINVAL, "%s: NULL pointer in chunk %d", what, k);
        if (!aligned(d_master[k], 4) || !aligned(d_exp_avg[k], 4) || !aligned(d_exp_avg_sq[k], 4) || !aligned(g, bf16 ? 2 : 4) ||
            (d_param_bf16 && !aligned(d_param_bf16[k], 2)))
            return fail(ELIXIR_EALIGN, "%s: a pointer of chunk %d is not aligned for its element type", what, k);
        if (d_param_bf16 && !d_param_bf16[k]) return fail(ELIXIR_EINVAL, "%s: d_param_bf16[%d] is NULL", what, k);
    }
    const AdamConsts c = make_consts(hp);
    hipStream_t s = (hipStream_t)stream;
    const bool has_out = d_param_bf16 != nullptr;
    AdamMultiTable tab;
    int in_table = 0;
    int64_t max_blocks = 0, used_blocks = 0;  // grid row length; workgroups that have work
    auto flush = [&]() -> int {
        if (in_table == 0) return ELIXIR_OK;
        for (int j = in_table; j < kAdamMultiMax; ++j) {
            tab.master[j] = tab.exp_avg[j] = tab.exp_avg_sq[j] = nullptr;
            tab.grad[j] = nullptr;
            tab.out[j] = nullptr;
            tab.n2[j] = 0;
        }
        const dim3 grid((unsigned)max_blocks, (unsigned)in_table), block(kAdamBlock);
        if (bf16) {
            if (has_out) hipLaunchKernelGGL((adam_multi_kernel<true, true>), grid, block, kAdamLdsBytes, s, tab, c, d_grad_scale);
            else hipLaunchKernelGGL((adam_multi_kernel<true, false>), grid, block, kAdamLdsBytes, s, tab, c, d_grad_scale);
        } else {
            if (has_out) hipLaunchKernelGGL((adam_multi_kernel<false, true>), grid, block, kAdamLdsBytes, s, tab, c, d_grad_scale);
            else hipLaunchKernelGGL((adam_multi_kernel<false, false>), grid, block, kAdamLdsBytes, s, tab, c, d_grad_scale);
        }
        ELIXIR_LAUNCH_CHECK("adam_multi_kernel");
        in_table = 0;
        max_blocks = used_blocks = 0;
        return ELIXIR_OK;
    };
    for (int k = 0; k < n_chunks; ++k) {
        if (n[k] == 0) continue;
        const void* g = bf16 ? (const void*)d_grad_bf16[k] : (const void*)d_grad_fp32[k];
        uint16_t* out = has_out ? d_param_bf16[k] : nullptr;
        const int head = phase(d_master[k], 4);
        const bool vec = head == 0 && phase(d_exp_avg[k], 4) == 0 && phase(d_exp_avg_sq[k], 4) == 0 &&
                         phase(g, bf16 ? 2 : 4) == 0 && (!out || phase(out, 2) == 0) && n[k] >= kAdamVec;
        const int64_t pairs = vec ? n[k] / kAdamVec : 0;
        const int64_t nb = (pairs + kAdamBlock - 1) / kAdamBlock;
        if (!vec || nb > kMaxBlocksPerLaunch) {
            // a slice at an odd offset, or a chunk too long for one grid row: the single-chunk path
            if (const int rc = flush()) return rc;
            if (const int rc = elixir_chunk_adam_step(d_master[k], d_exp_avg[k], d_exp_avg_sq[k], bf16 ? nullptr : d_grad_fp32[k],
                                                      bf16 ? d_grad_bf16[k] : nullptr, out, n[k], hp, d_grad_scale, stream))
                return rc;
            continue;
        }
        // every chunk gets a grid row as long as the longest one: start a new launch when the table is full or
        // when rows of very different length would leave more than ~a quarter of the workgroups without work
        const int64_t row = nb > max_blocks ? nb : max_blocks;
        const bool wasteful = row * (in_table + 1) - (used_blocks + nb) > (used_blocks + nb) / 4 + 1024;
        if (in_table == kAdamMultiMax || (in_table > 0 && wasteful))
            if (const int rc = flush()) return rc;
        const int j = in_table++;
        tab.master[j] = d_master[k];
        tab.exp_avg[j] = d_exp_avg[k];
        tab.exp_avg_sq[j] = d_exp_avg_sq[k];
        tab.grad[j] = g;
        tab.out[j] = out;
        tab.n2[j] = pairs;
        if (nb > max_blocks) max_blocks = nb;
        used_blocks += nb;
        if (n[k] % kAdamVec) {  // the odd last element of this chunk
            if (bf16) launch_scalar<true>(d_master[k], d_exp_avg[k], d_exp_avg_sq[k], g, out, pairs * kAdamVec, n[k], c, d_grad_scale, s);
            else launch_scalar<false>(d_master[k], d_exp_avg[k], d_exp_avg_sq[k], g, out, pairs * kAdamVec, n[k], c, d_grad_scale, s);
            ELIXIR_LAUNCH_CHECK("adam_scalar_kernel");
        }
    }
    return flush();
}
