// elixir_host_adam_step: the AdamW update of a host-resident chunk on the host cores.
//
// In the paper a chunk whose optimizer chunk lives in CPU memory is updated by the CPU: only the
// low-precision gradients travel to the host and only the new low-precision parameters travel back
// (Sec. 2 "Memory Offloading"; the CPU update velocity V_c of Sec. 5 and App. B).  This is that update:
// the same per-element arithmetic as the GPU kernel (fp32, fused multiply-adds where the GPU has them;
// square root and division are the correctly rounded IEEE ones here), vectorised for AVX-512 or AVX2
// with a scalar fallback chosen at run time, and spread over host threads in contiguous slices.
// Per element 14 bytes are read and 14 written in host memory; new values leave the cache with
// non-temporal stores where the slice is 64-byte aligned.
#include <immintrin.h>
#include <math.h>
#include <sched.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <thread>
#include <vector>

#include "status.hpp"

using namespace elixir;

namespace {

struct Consts {
    float lr_wd, beta1, omb1, beta2, omb2, step_size, inv_sqrt_bc2, eps, grad_scale;
};

inline float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

inline uint16_t f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// fp16 (IEEE binary16: 1 sign, 5 exponent, 10 fraction bits) for the scalar path, written out on the bit patterns;
// the vector paths use the CPU's conversion instructions, which compute the same.  Widening is exact.
inline float f16_to_f32(uint16_t b) {
    const uint32_t sign = (uint32_t)(b & 0x8000u) << 16;
    uint32_t exp = (b >> 10) & 0x1Fu, frac = b & 0x3FFu, u;
    if (exp == 0x1Fu) {
        u = sign | 0x7F800000u | (frac << 13);  // Inf, or NaN with its payload
    } else if (exp != 0) {
        u = sign | ((exp + 112u) << 23) | (frac << 13);
    } else if (frac == 0) {
        u = sign;
    } else {  // subnormal: frac * 2^-24, normalised
        int e = 113;
        while (!(frac & 0x400u)) {
            frac <<= 1;
            --e;
        }
        u = sign | ((uint32_t)e << 23) | ((frac & 0x3FFu) << 13);
    }
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// Narrowing rounds to nearest, ties to even; values beyond the largest finite fp16 become Inf; NaN stays a quiet NaN.
inline uint16_t f32_to_f16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((a >> 13) & 0x3FFu));
    if (a >= 0x38800000u) {  // at least 2^-14: a normal fp16, unless it rounds up to Inf
        const uint32_t r = a + 0xFFFu + ((a >> 13) & 1u);
        const uint32_t h = (r - 0x38000000u) >> 13;
        return (uint16_t)(sign | (h > 0x7C00u ? 0x7C00u : h));
    }
    if (a < 0x33000000u) return sign;  // below 2^-25: rounds to zero (2^-25 itself is a tie and goes to the even 0)
    const uint32_t m = (a & 0x7FFFFFu) | 0x800000u;
    const uint32_t shift = 126u - (a >> 23);  // 14 .. 24
    const uint32_t lsb = (m >> shift) & 1u;
    return (uint16_t)(sign | ((m + ((1u << (shift - 1)) - 1u) + lsb) >> shift));
}

template <bool FP16>
void adam_scalar(float* p, float* m, float* v, const float* g32, const uint16_t* g16, uint16_t* out, int64_t n,
                 const Consts& c) {
    for (int64_t k = 0; k < n; ++k) {
        const float g = c.grad_scale * (g32 ? g32[k] : FP16 ? f16_to_f32(g16[k]) : bf16_to_f32(g16[k]));
        const float mk = fmaf(c.beta1, m[k], c.omb1 * g);
        const float vk = fmaf(c.beta2, v[k], (c.omb2 * g) * g);
        const float denom = fmaf(sqrtf(vk), c.inv_sqrt_bc2, c.eps);
        const float upd = (c.step_size * mk) / denom;
        const float pk = p[k] + fmaf(p[k], -c.lr_wd, -upd);
        p[k] = pk;
        m[k] = mk;
        v[k] = vk;
        if (out) out[k] = FP16 ? f32_to_f16(pk) : f32_to_bf16(pk);
    }
}

template <bool FP16>
__attribute__((target("avx2,fma,f16c"))) void adam_avx2(float* p, float* m, float* v, const float* g32, const uint16_t* g16,
                                                       uint16_t* out, int64_t n, const Consts& c) {
    const __m256 b1 = _mm256_set1_ps(c.beta1), o1 = _mm256_set1_ps(c.omb1), b2 = _mm256_set1_ps(c.beta2),
                 o2 = _mm256_set1_ps(c.omb2), ss = _mm256_set1_ps(c.step_size), ib = _mm256_set1_ps(c.inv_sqrt_bc2),
                 eps = _mm256_set1_ps(c.eps), nlw = _mm256_set1_ps(-c.lr_wd), gs = _mm256_set1_ps(c.grad_scale);
    int64_t k = 0;
    for (; k + 8 <= n; k += 8) {
        __m256 g;
        if (g32) g = _mm256_loadu_ps(g32 + k);
        else if (FP16) g = _mm256_cvtph_ps(_mm_loadu_si128((const __m128i*)(g16 + k)));
        else g = _mm256_castsi256_ps(_mm256_slli_epi32(_mm256_cvtepu16_epi32(_mm_loadu_si128((const __m128i*)(g16 + k))), 16));
        g = _mm256_mul_ps(gs, g);
        const __m256 pk0 = _mm256_loadu_ps(p + k);
        const __m256 mk = _mm256_fmadd_ps(b1, _mm256_loadu_ps(m + k), _mm256_mul_ps(o1, g));
        const __m256 vk = _mm256_fmadd_ps(b2, _mm256_loadu_ps(v + k), _mm256_mul_ps(_mm256_mul_ps(o2, g), g));
        const __m256 denom = _mm256_fmadd_ps(_mm256_sqrt_ps(vk), ib, eps);
        const __m256 upd = _mm256_div_ps(_mm256_mul_ps(ss, mk), denom);
        // -(lr*wd)*p - upd
        const __m256 pk = _mm256_add_ps(pk0, _mm256_fmsub_ps(pk0, nlw, upd));
        _mm256_storeu_ps(p + k, pk);
        _mm256_storeu_ps(m + k, mk);
        _mm256_storeu_ps(v + k, vk);
        if (out && FP16) {
            _mm_storeu_si128((__m128i*)(out + k), _mm256_cvtps_ph(pk, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC));
        } else if (out) {
            const __m256i u = _mm256_castps_si256(pk);
            const __m256i lsb = _mm256_and_si256(_mm256_srli_epi32(u, 16), _mm256_set1_epi32(1));
            __m256i r = _mm256_srli_epi32(_mm256_add_epi32(_mm256_add_epi32(u, _mm256_set1_epi32(0x7FFF)), lsb), 16);
            const __m256i is_nan = _mm256_cmpgt_epi32(_mm256_and_si256(u, _mm256_set1_epi32(0x7FFFFFFF)), _mm256_set1_epi32(0x7F800000));
            const __m256i nan_bits = _mm256_or_si256(_mm256_srli_epi32(u, 16), _mm256_set1_epi32(0x40));
            r = _mm256_blendv_epi8(r, nan_bits, is_nan);
            const __m256i packed = _mm256_permute4x64_epi64(_mm256_packus_epi32(r, r), 0xD8);
            _mm_storeu_si128((__m128i*)(out + k), _mm256_castsi256_si128(packed));
        }
    }
    if (k < n) adam_scalar<FP16>(p + k, m + k, v + k, g32 ? g32 + k : nullptr, g16 ? g16 + k : nullptr, out ? out + k : nullptr, n - k, c);
}

template <bool FP16>
__attribute__((target("avx512f,avx512bw,avx512vl"))) void adam_avx512(float* p, float* m, float* v, const float* g32,
                                                                     const uint16_t* g16, uint16_t* out, int64_t n,
                                                                     const Consts& c) {
    const __m512 b1 = _mm512_set1_ps(c.beta1), o1 = _mm512_set1_ps(c.omb1), b2 = _mm512_set1_ps(c.beta2),
                 o2 = _mm512_set1_ps(c.omb2), ss = _mm512_set1_ps(c.step_size), ib = _mm512_set1_ps(c.inv_sqrt_bc2),
                 eps = _mm512_set1_ps(c.eps), nlw = _mm512_set1_ps(-c.lr_wd), gs = _mm512_set1_ps(c.grad_scale);
    // leading elements up to the first 64-byte boundary of p, so that the streaming stores are aligned
    int64_t head = (int64_t)(((64 - ((uintptr_t)p & 63)) & 63) / 4);
    if (head > n) head = n;
    if (head) adam_scalar<FP16>(p, m, v, g32, g16, out, head, c);
    const bool stream = (((uintptr_t)(m + head) | (uintptr_t)(v + head)) & 63) == 0;
    const bool stream_out = out && (((uintptr_t)(out + head)) & 31) == 0;
    int64_t k = head;
    for (; k + 16 <= n; k += 16) {
        __m512 g;
        if (g32) g = _mm512_loadu_ps(g32 + k);
        else if (FP16) g = _mm512_cvtph_ps(_mm256_loadu_si256((const __m256i*)(g16 + k)));
        else g = _mm512_castsi512_ps(_mm512_slli_epi32(_mm512_cvtepu16_epi32(_mm256_loadu_si256((const __m256i*)(g16 + k))), 16));
        g = _mm512_mul_ps(gs, g);
        const __m512 pk0 = _mm512_load_ps(p + k);
        const __m512 mk = _mm512_fmadd_ps(b1, _mm512_loadu_ps(m + k), _mm512_mul_ps(o1, g));
        const __m512 vk = _mm512_fmadd_ps(b2, _mm512_loadu_ps(v + k), _mm512_mul_ps(_mm512_mul_ps(o2, g), g));
        const __m512 denom = _mm512_fmadd_ps(_mm512_sqrt_ps(vk), ib, eps);
        const __m512 upd = _mm512_div_ps(_mm512_mul_ps(ss, mk), denom);
        const __m512 pk = _mm512_add_ps(pk0, _mm512_fmsub_ps(pk0, nlw, upd));
        if (stream) {
            _mm512_stream_ps(p + k, pk);
            _mm512_stream_ps(m + k, mk);
            _mm512_stream_ps(v + k, vk);
        } else {
            _mm512_store_ps(p + k, pk);
            _mm512_storeu_ps(m + k, mk);
            _mm512_storeu_ps(v + k, vk);
        }
        if (out && FP16) {
            const __m256i packed = _mm512_cvtps_ph(pk, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
            if (stream_out) _mm256_stream_si256((__m256i*)(out + k), packed);
            else _mm256_storeu_si256((__m256i*)(out + k), packed);
        } else if (out) {
            const __m512i u = _mm512_castps_si512(pk);
            const __m512i lsb = _mm512_and_si512(_mm512_srli_epi32(u, 16), _mm512_set1_epi32(1));
            __m512i r = _mm512_srli_epi32(_mm512_add_epi32(_mm512_add_epi32(u, _mm512_set1_epi32(0x7FFF)), lsb), 16);
            const __mmask16 is_nan = _mm512_cmpgt_epi32_mask(_mm512_and_si512(u, _mm512_set1_epi32(0x7FFFFFFF)), _mm512_set1_epi32(0x7F800000));
            r = _mm512_mask_mov_epi32(r, is_nan, _mm512_or_si512(_mm512_srli_epi32(u, 16), _mm512_set1_epi32(0x40)));
            const __m256i packed = _mm512_cvtepi32_epi16(r);
            if (stream_out) _mm256_stream_si256((__m256i*)(out + k), packed);
            else _mm256_storeu_si256((__m256i*)(out + k), packed);
        }
    }
    _mm_sfence();
    if (k < n) adam_scalar<FP16>(p + k, m + k, v + k, g32 ? g32 + k : nullptr, g16 ? g16 + k : nullptr, out ? out + k : nullptr, n - k, c);
}

typedef void (*AdamFn)(float*, float*, float*, const float*, const uint16_t*, uint16_t*, int64_t, const Consts&);

// Best instruction set the CPU offers; the environment variable ELIXIR_HOST_ISA (scalar | avx2 | avx512) can only
// lower the choice (used by tests to exercise every variant on one machine).
AdamFn pick_kernel(const char** name, bool fp16 = false) {
    __builtin_cpu_init();
    int level = 0;
    if (__builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma") && __builtin_cpu_supports("f16c")) level = 1;
    if (level == 1 && __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512vl")) level = 2;
    if (const char* want = getenv("ELIXIR_HOST_ISA")) {
        const int cap = !strcmp(want, "scalar") ? 0 : !strcmp(want, "avx2") ? 1 : 2;
        if (cap < level) level = cap;
    }
    if (level == 2) {
        *name = "avx512";
        return fp16 ? adam_avx512<true> : adam_avx512<false>;
    }
    if (level == 1) {
        *name = "avx2";
        return fp16 ? adam_avx2<true> : adam_avx2<false>;
    }
    *name = "scalar";
    return fp16 ? adam_scalar<true> : adam_scalar<false>;
}

int available_cores() {
    cpu_set_t set;
    if (sched_getaffinity(0, sizeof(set), &set) == 0) {
        const int n = CPU_COUNT(&set);
        if (n > 0) return n;
    }
    const unsigned h = std::thread::hardware_concurrency();
    return h ? (int)h : 1;
}

}  // namespace

extern "C" const char* elixir_host_adam_isa(void) {
    const char* name = "";
    (void)pick_kernel(&name);
    return name;
}

namespace {

int check_hparams_host(const char* what, int64_t n, const elixir_adam_hparams* hp) {
    if (n < 0) return fail(ELIXIR_EINVAL, "%s: n=%lld is negative", what, (long long)n);
    if (!hp) return fail(ELIXIR_EINVAL, "%s: hp is NULL", what);
    if (hp->step < 1) return fail(ELIXIR_EINVAL, "%s: step=%lld, steps count from 1", what, (long long)hp->step);
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(ELIXIR_EINVAL, "%s: betas must lie in [0, 1)", what);
    if (!(hp->eps >= 0.0f) || !isfinite(hp->lr) || !isfinite(hp->weight_decay))
        return fail(ELIXIR_EINVAL, "%s: eps must be >= 0 and lr, weight_decay finite", what);
    return ELIXIR_OK;
}

Consts make_consts(const elixir_adam_hparams* hp, float grad_scale) {
    const double lr = hp->lr, b1 = hp->beta1, b2 = hp->beta2;
    const double bc1 = 1.0 - pow(b1, (double)hp->step), bc2 = 1.0 - pow(b2, (double)hp->step);
    Consts c;
    c.lr_wd = (float)(lr * (double)hp->weight_decay);
    c.beta1 = hp->beta1;
    c.omb1 = (float)(1.0 - b1);
    c.beta2 = hp->beta2;
    c.omb2 = (float)(1.0 - b2);
    c.step_size = (float)(lr / bc1);
    c.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
    c.eps = hp->eps;
    c.grad_scale = grad_scale;
    return c;
}

// Runs work(t) for t = 0 .. T-1 on T threads (the caller's thread takes t = 0).
template <typename W>
int run_threads(const char* what, int T, W&& work) {
    if (T == 1) {
        work(0);
        return ELIXIR_OK;
    }
    std::vector<std::thread> pool;
    try {
        pool.reserve(T - 1);
        for (int t = 1; t < T; ++t) pool.emplace_back(work, t);
    } catch (...) {
        for (auto& th : pool) th.join();
        return fail(ELIXIR_EINVAL, "%s: could not start %d threads", what, T);
    }
    work(0);
    for (auto& th : pool) th.join();
    return ELIXIR_OK;
}

}  // namespace

extern "C" int elixir_host_adam_step_lp(float* h_master, float* h_exp_avg, float* h_exp_avg_sq, const float* h_grad_fp32,
                                        const uint16_t* h_grad_bf16, uint16_t* h_param_bf16, int lowp_format, int64_t n,
                                        const elixir_adam_hparams* hp, float grad_scale, int n_threads) {
    static const char* what = "elixir_host_adam_step";
    if (const int rc = check_hparams_host(what, n, hp)) return rc;
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (n == 0) return ELIXIR_OK;
    if ((h_grad_fp32 != nullptr) == (h_grad_bf16 != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of h_grad_fp32 / h_grad_bf16 must be given", what);
    if (!h_master || !h_exp_avg || !h_exp_avg_sq) return fail(ELIXIR_EINVAL, "%s: master / exp_avg / exp_avg_sq must not be NULL", what);
    const uintptr_t a4 = (uintptr_t)h_master | (uintptr_t)h_exp_avg | (uintptr_t)h_exp_avg_sq | (uintptr_t)h_grad_fp32;
    const uintptr_t a2 = (uintptr_t)h_grad_bf16 | (uintptr_t)h_param_bf16;
    if ((a4 & 3) || (a2 & 1)) return fail(ELIXIR_EALIGN, "%s: a pointer is not aligned for its element type", what);
    const Consts c = make_consts(hp, grad_scale);
    const char* isa;
    const AdamFn fn = pick_kernel(&isa, lowp_format == ELIXIR_LOWP_FP16);
    int T = n_threads > 0 ? n_threads : available_cores();
    const int64_t min_slice = 1 << 16;  // below this a thread costs more than it saves
    if ((int64_t)T > (n + min_slice - 1) / min_slice) T = (int)((n + min_slice - 1) / min_slice);
    if (T < 1) T = 1;
    // contiguous slices, boundaries on multiples of 16 elements so that every slice but the first starts 64-byte
    // aligned relative to the chunk
    auto bound = [&](int t) -> int64_t {
        if (t >= T) return n;
        return (n / T * t) & ~(int64_t)15;
    };
    return run_threads(what, T, [&](int t) {
        const int64_t a = bound(t), b = bound(t + 1);
        if (a < b)
            fn(h_master + a, h_exp_avg + a, h_exp_avg_sq + a, h_grad_fp32 ? h_grad_fp32 + a : nullptr,
               h_grad_bf16 ? h_grad_bf16 + a : nullptr, h_param_bf16 ? h_param_bf16 + a : nullptr, b - a, c);
    });
}

// The same update on a tiled optimizer chunk ([master tile | m tile | v tile] of ELIXIR_STATE_TILE elements each): a
// chunk that the plan moves between host and device is then updated in place by either side.  Threads take whole tiles.
extern "C" int elixir_host_adam_step(float* h_master, float* h_exp_avg, float* h_exp_avg_sq, const float* h_grad_fp32,
                                     const uint16_t* h_grad_bf16, uint16_t* h_param_bf16, int64_t n,
                                     const elixir_adam_hparams* hp, float grad_scale, int n_threads) {
    return elixir_host_adam_step_lp(h_master, h_exp_avg, h_exp_avg_sq, h_grad_fp32, h_grad_bf16, h_param_bf16, ELIXIR_LOWP_BF16, n, hp,
                                    grad_scale, n_threads);
}

extern "C" int elixir_host_adam_step_tiled_lp(float* h_state, const float* h_grad_fp32, const uint16_t* h_grad_bf16,
                                              uint16_t* h_param_bf16, int lowp_format, int64_t n, const elixir_adam_hparams* hp,
                                              float grad_scale, int n_threads) {
    static const char* what = "elixir_host_adam_step_tiled";
    if (const int rc = check_hparams_host(what, n, hp)) return rc;
    if (lowp_format != ELIXIR_LOWP_BF16 && lowp_format != ELIXIR_LOWP_FP16)
        return fail(ELIXIR_EINVAL, "%s: lowp_format=%d is neither ELIXIR_LOWP_BF16 nor ELIXIR_LOWP_FP16", what, lowp_format);
    if (n == 0) return ELIXIR_OK;
    if ((h_grad_fp32 != nullptr) == (h_grad_bf16 != nullptr))
        return fail(ELIXIR_EINVAL, "%s: exactly one of h_grad_fp32 / h_grad_bf16 must be given", what);
    if (!h_state) return fail(ELIXIR_EINVAL, "%s: h_state is NULL", what);
    if ((((uintptr_t)h_state | (uintptr_t)h_grad_fp32) & 3) || (((uintptr_t)h_grad_bf16 | (uintptr_t)h_param_bf16) & 1))
        return fail(ELIXIR_EALIGN, "%s: a pointer is not aligned for its element type", what);
    const Consts c = make_consts(hp, grad_scale);
    const char* isa;
    const AdamFn fn = pick_kernel(&isa, lowp_format == ELIXIR_LOWP_FP16);
    constexpr int64_t kTile = ELIXIR_STATE_TILE;
    const int64_t tiles = (n + kTile - 1) / kTile;
    int T = n_threads > 0 ? n_threads : available_cores();
    if ((int64_t)T > (tiles + 15) / 16) T = (int)((tiles + 15) / 16);   // at least 16 tiles (64Ki elements) per thread
    if (T < 1) T = 1;
    return run_threads(what, T, [&](int t) {
        const int64_t t0 = tiles * t / T, t1 = tiles * (t + 1) / T;
        for (int64_t i = t0; i < t1; ++i) {
            const int64_t e = i * kTile, cnt = n - e < kTile ? n - e : kTile;
            float* base = h_state + 3 * kTile * i;
            fn(base, base + kTile, base + 2 * kTile, h_grad_fp32 ? h_grad_fp32 + e : nullptr, h_grad_bf16 ? h_grad_bf16 + e : nullptr,
               h_param_bf16 ? h_param_bf16 + e : nullptr, cnt, c);
        }
    });
}

extern "C" int elixir_host_adam_step_tiled(float* h_state, const float* h_grad_fp32, const uint16_t* h_grad_bf16,
                                           uint16_t* h_param_bf16, int64_t n, const elixir_adam_hparams* hp, float grad_scale,
                                           int n_threads) {
    return elixir_host_adam_step_tiled_lp(h_state, h_grad_fp32, h_grad_bf16, h_param_bf16, ELIXIR_LOWP_BF16, n, hp, grad_scale, n_threads);
}
