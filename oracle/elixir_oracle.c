/*
 * CPU oracle for the chunked mixed-precision AdamW step (TEST INFRASTRUCTURE).
 *
 * Plain, slow, scalar C.  Every floating-point result is computed in double
 * precision from the stored inputs and rounded ONCE to its storage type
 * (fp32 for master weights, moments and gradient chunks; bf16 for the
 * low-precision parameter copy).  Nothing here is blocked, fused, vectorised
 * by hand or shared with the GPU library; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * What each function follows:
 *   - chunk = a group of parameters flattened and concatenated into one
 *     fixed-length 1-D buffer (paper Sec. 3, "Chunk"; Fig. 3 left);
 *   - mixed precision: low-precision parameters and gradients, fp32 master
 *     weight + Adam moments (12 bytes/param), master rounded to low precision
 *     after the update (paper Sec. 2, "Mixed Precision Training");
 *   - one optimizer update consumes a gradient chunk and its optimizer chunk
 *     (paper Sec. 4.1);
 *   - Adam as in Kingma & Ba Alg. 1 with the decoupled weight decay of
 *     Loshchilov & Hutter Alg. 2 (the paper cites Adam and prints no update
 *     rule; eps is added after bias-correcting sqrt(v)).
 * The global gradient norm and clipping are not in the paper; they follow the
 * usual definition  coef = min(1, max_norm / (norm + 1e-6)).
 *
 * The low-precision format is bf16 in the benchmark configurations and fp16 in the paper; both are here
 * (fmt 0 / 1).  With fp16 the caller scales the loss; the unscaling is part of grad_scale.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

/* bf16 is the upper half of an fp32 pattern: widening appends 16 zero bits. */
float orc_bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Round to nearest, ties to even, on the fp32 bit pattern.  NaN stays a quiet
 * NaN; +-Inf is preserved; finite values above the largest bf16 round to Inf. */
uint16_t orc_f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

void orc_bf16_to_f32_array(const uint16_t* in, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_to_f32(in[i]);
}
void orc_f32_to_bf16_array(const float* in, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f32_to_bf16_rne(in[i]);
}

/* ---- fp16 <-> fp32 (the paper's low-precision format; IEEE binary16) ------ */

float orc_f16_to_f32(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const int exp = (h >> 10) & 0x1F;
    const uint32_t man = h & 0x3FFu;
    double v;
    if (exp == 31) {
        uint32_t u = sign | 0x7F800000u | (man << 13);
        float f;
        memcpy(&f, &u, 4);
        return f;
    }
    if (exp == 0) v = ldexp((double)man, -24);              /* subnormal: man * 2^-24 */
    else v = ldexp(1.0 + (double)man / 1024.0, exp - 15);
    return (float)(sign ? -v : v);
}

/* Round to nearest, ties to even, by construction: scale into the fp16 grid, round with the double
 * rounding-free nearbyint (default rounding mode is to-nearest-even), rebuild the pattern. */
uint16_t orc_f32_to_f16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);            /* NaN -> quiet NaN */
    double a = fabs((double)f);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    int e;
    (void)frexp(a, &e);                       /* a = frac * 2^e, frac in [0.5, 1) -> a in [2^(e-1), 2^e) */
    int ex = e - 1;                           /* exponent of the leading bit */
    if (ex < -14) ex = -14;                   /* subnormal range: fixed grid of 2^-24 */
    const double grid = ldexp(1.0, ex - 10);  /* spacing of fp16 values in this binade */
    const double q = nearbyint(a / grid);     /* exact division by a power of two, then ties-to-even */
    const double r = q * grid;
    if (r >= 65520.0) return (uint16_t)(sign | 0x7C00u);    /* rounds past the largest finite value (65504) */
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)q);        /* subnormal: q = mantissa */
    int e2;
    const double fr = frexp(r, &e2);          /* r = fr * 2^e2, fr in [0.5,1) */
    const int bexp = e2 - 1 + 15;
    const uint16_t man = (uint16_t)((fr * 2.0 - 1.0) * 1024.0);
    return (uint16_t)(sign | (bexp << 10) | man);
}

void orc_f16_to_f32_array(const uint16_t* in, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f16_to_f32(in[i]);
}
void orc_f32_to_f16_array(const float* in, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f32_to_f16_rne(in[i]);
}

/* low-precision format selector: 0 = bf16, 1 = fp16 */
static float orc_lowp_to_f32(uint16_t b, int fmt) { return fmt ? orc_f16_to_f32(b) : orc_bf16_to_f32(b); }
static uint16_t orc_f32_to_lowp(float f, int fmt) { return fmt ? orc_f32_to_f16_rne(f) : orc_f32_to_bf16_rne(f); }

/* ---- pack / unpack ------------------------------------------------------ */

/* chunk[offset_i + k] = tensor_i[k]; every byte not covered by a tensor is 0. */
void orc_chunk_pack(void* chunk, int64_t chunk_elems, int elem_size, const void* const* tensors,
                    const int64_t* numel, const int64_t* offset, int T) {
    memset(chunk, 0, (size_t)chunk_elems * (size_t)elem_size);
    for (int i = 0; i < T; ++i)
        memcpy((char*)chunk + (size_t)offset[i] * elem_size, tensors[i], (size_t)numel[i] * elem_size);
}

/* tensor_i[k] = chunk[offset_i + k]. */
void orc_chunk_unpack(const void* chunk, int64_t chunk_elems, int elem_size, void* const* tensors,
                      const int64_t* numel, const int64_t* offset, int T) {
    (void)chunk_elems;
    for (int i = 0; i < T; ++i)
        memcpy(tensors[i], (const char*)chunk + (size_t)offset[i] * elem_size, (size_t)numel[i] * elem_size);
}

/* ---- gradient reduction into the fp32 chunk ----------------------------- */

/* gchunk[offset+k] = fl32( (accumulate ? gchunk[offset+k] : 0) + fl32(scale * g[k]) ).
 * On one GPU "reduce" is the accumulation of micro-batch gradients (the
 * cross-rank reduce of the paper's Sec. 2 / Fig. 3 right has one rank). */
void orc_grad_reduce_into_chunk_lp(float* gchunk, int64_t offset, const uint16_t* g_lowp, int fmt, int64_t n,
                                   float scale, int accumulate) {
    for (int64_t k = 0; k < n; ++k) {
        float t = (float)((double)scale * (double)orc_lowp_to_f32(g_lowp[k], fmt)); /* fl32(scale*g): a 24-bit times an at most 11-bit significand is exact in double */
        float old = accumulate ? gchunk[offset + k] : 0.0f;
        gchunk[offset + k] = (float)((double)old + (double)t);
    }
}
void orc_grad_reduce_into_chunk(float* gchunk, int64_t offset, const uint16_t* g_bf16, int64_t n, float scale,
                                int accumulate) {
    orc_grad_reduce_into_chunk_lp(gchunk, offset, g_bf16, 0, n, scale, accumulate);
}

/* ---- global L2 norm ----------------------------------------------------- */

/* sum of squares of n fp32 values, sequentially, in double. */
double orc_sum_squares(const float* g, int64_t n) {
    double s = 0.0;
    for (int64_t k = 0; k < n; ++k) s += (double)g[k] * (double)g[k];
    return s;
}

/* coef = min(1, max_norm / (norm + 1e-6)); max_norm <= 0 means no clipping. */
double orc_clip_coef(double norm, double max_norm) {
    if (!(max_norm > 0.0)) return 1.0;
    double c = max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ---- AdamW over one chunk ----------------------------------------------- */

/* One decoupled-weight-decay Adam step on n elements.
 *   g = grad_scale * grad          (grad from the fp32 chunk, or bf16 widened)
 *   p = p * (1 - lr*wd)
 *   m = b1*m + (1-b1)*g            v = b2*v + (1-b2)*g*g
 *   p = p - lr * (m/(1-b1^t)) / ( sqrt(v/(1-b2^t)) + eps )
 *   store fl32(p), fl32(m), fl32(v);  out = bf16_rne(fl32(p))
 * Exactly one of grad_f32 / grad_bf16 is non-NULL; param_bf16 may be NULL.
 * step is 1-based. */
void orc_chunk_adam_step_lp(float* master, float* exp_avg, float* exp_avg_sq, const float* grad_f32,
                            const uint16_t* grad_bf16, uint16_t* param_bf16, int fmt, int64_t n, float lr_f,
                            float beta1_f, float beta2_f, float eps_f, float wd_f, int64_t step, double grad_scale) {
    const double lr = lr_f, b1 = beta1_f, b2 = beta2_f, eps = eps_f, wd = wd_f;
    const double bc1 = 1.0 - pow(b1, (double)step);
    const double bc2 = 1.0 - pow(b2, (double)step);
    for (int64_t k = 0; k < n; ++k) {
        double g = grad_scale * (grad_f32 ? (double)grad_f32[k] : (double)orc_lowp_to_f32(grad_bf16[k], fmt));
        double p = (double)master[k] * (1.0 - lr * wd);
        double m = b1 * (double)exp_avg[k] + (1.0 - b1) * g;
        double v = b2 * (double)exp_avg_sq[k] + (1.0 - b2) * g * g;
        p = p - lr * (m / bc1) / (sqrt(v / bc2) + eps);
        float pf = (float)p;
        master[k] = pf;
        exp_avg[k] = (float)m;
        exp_avg_sq[k] = (float)v;
        if (param_bf16) param_bf16[k] = orc_f32_to_lowp(pf, fmt);
    }
}
void orc_chunk_adam_step(float* master, float* exp_avg, float* exp_avg_sq, const float* grad_f32,
                         const uint16_t* grad_bf16, uint16_t* param_bf16, int64_t n, float lr_f, float beta1_f,
                         float beta2_f, float eps_f, float wd_f, int64_t step, double grad_scale) {
    orc_chunk_adam_step_lp(master, exp_avg, exp_avg_sq, grad_f32, grad_bf16, param_bf16, 0, n, lr_f, beta1_f, beta2_f, eps_f,
                           wd_f, step, grad_scale);
}
