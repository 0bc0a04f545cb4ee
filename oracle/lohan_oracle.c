/*
 * CPU oracle for the per-block mixed-precision Adam/AdamW step of LoHan's active gradient
 * offloading.  THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares nothing with the HIP path.
 *
 * What the paper fixes (LoHan, arxiv 2403.06504):
 *   - Sec. IV-C, "Naive Active Gradient Offloading": when gradient tensor i arrives, the
 *     "CPU Compute" step updates the model states of tensor i and produces a 16-bit parameter
 *     copy.  This file is that step for one flat tensor/block.
 *   - Table II: the tensors and their widths -- P32 (4 B/param), OS32 (8 B/param, here the two
 *     Adam moments m and v), G16 (2 B/param), P16 (2 B/param).
 *   - Sec. II, "LLM Training Stages": the optimizer is Adam (Kingma & Ba, Algorithm 1).
 *   - Sec. V-A, "Workloads": training is in mixed precision.
 *   - Sec. IV-C, footnote: the update is synchronous; forward/backward read the updated model,
 *     hence P16 is always the rounding of the P32 written by the same step.
 * The paper never writes the update down.  Everything else (loss-scale unscale, inf/nan skip,
 * AdamW decoupled decay, eps outside the square root after bias correction, bf16 round-to-nearest-
 * even, operation order) is a reading of the paper, stated here step by step where it is used.
 *
 * Precision: the state is fp32 by Table II and the parity bar is in fp32 ulps after ten chained
 * steps, so the step is evaluated in fp32, one IEEE-754 operation at a time, each rounded to
 * nearest-even, in the fixed order written below; no fused multiply-add, gradual underflow.
 * Build with -O2 -ffp-contract=off -fno-fast-math on x86-64 (SSE scalar arithmetic; sqrtf and '/'
 * are correctly rounded).  A float64 evaluation of the textbook formula lives in textbook_f64.py
 * and is used only to pin this file.
 *
 * Every function below is pinned by tests/test_oracle_pins.py (closed-form first step, hand
 * examples under tests/golden/, exact rational re-evaluation, float64 textbook formula, a library
 * AdamW, invariants).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- number formats --------------------------------------------------------------------- */

/* IEEE binary16 bit pattern -> fp32 value (exact: every binary16 value is an fp32 value).
 * G16 is 2 bytes per parameter (Table II); the reading takes it as IEEE half precision. */
static float half_bits_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t frac = (uint32_t)h & 0x3FFu;
    float mag;
    if (expo == 0u) {
        mag = ldexpf((float)frac, -24);               /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 0x1Fu) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexpf((float)(frac | 0x400u), (int)expo - 25); /* (1024+frac) * 2^(e-15-10) */
    }
    return sign ? -mag : mag;
}

/* fp32 -> bfloat16 bit pattern, round to nearest, ties to even.  P16 is 2 bytes per parameter
 * (Table II) and is produced by the same step as the new P32 (Sec. IV-C). */
static uint16_t float_to_bf16_bits_rne(float x)
{
    uint32_t b;
    memcpy(&b, &x, sizeof b);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) {            /* NaN: keep sign and top payload, quiet */
        return (uint16_t)((b >> 16) | 0x0040u);
    }
    uint32_t lsb = (b >> 16) & 1u;
    b += 0x7FFFu + lsb;
    return (uint16_t)(b >> 16);
}

/* fp32 -> IEEE binary16 bit pattern, round to nearest, ties to even, overflow to infinity,
 * gradual underflow.  Used when the caller asks for an fp16 (instead of bf16) working copy: the
 * paper only says "16-bit parameter copy" (Sec. IV-C; P16 in Table II). */
static uint16_t float_to_half_bits_rne(float x)
{
    uint32_t b;
    memcpy(&b, &x, sizeof b);
    uint16_t sign = (uint16_t)((b >> 16) & 0x8000u);
    uint32_t a = b & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);          /* NaN -> quiet NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);         /* >= 65536 (and inf) */
    if (a >= 0x38800000u) {                                          /* >= 2^-14: normal half */
        uint32_t mant = a & 0x7FFFFFu;
        uint32_t h = (((a >> 23) - 112u) << 10) | (mant >> 13);      /* rebias 127 -> 15 */
        uint32_t rest = mant & 0x1FFFu;
        if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1u; /* may carry up to inf */
        return (uint16_t)(sign | h);
    }
    if (a <= 0x33000000u) return sign;                               /* <= 2^-25 rounds to zero */
    uint32_t mant = (a & 0x7FFFFFu) | 0x800000u;                     /* subnormal half: units of */
    uint32_t shift = 126u - (a >> 23);                               /* 2^-24                    */
    uint32_t h = mant >> shift;
    uint32_t rest = mant & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1u);
    if (rest > halfway || (rest == halfway && (h & 1u))) h += 1u;
    return (uint16_t)(sign | h);
}

/* ---- gradient overflow test ------------------------------------------------------------- */

/* 1 if any fp16 gradient of the block is +-inf or NaN (exponent field all ones), else 0.
 * The test is on the stored fp16 bits, before unscaling, over exactly the n elements given. */
int lohan_oracle_grad_overflow_check(const uint16_t *grad_fp16, uint64_t n)
{
    int flag = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if ((grad_fp16[i] & 0x7C00u) == 0x7C00u) flag = 1;
    }
    return flag;
}

/* Squared l2 norm of the unscaled gradients, sum_i (g16_i / loss_scale)^2, in float64, summed in
 * index order.  Used for per-block gradient clipping. */
double lohan_oracle_grad_sqnorm(const uint16_t *grad_fp16, uint64_t n, float loss_scale)
{
    double acc = 0.0;
    double s = (double)loss_scale;
    for (uint64_t i = 0; i < n; ++i) {
        double g = (double)half_bits_to_float(grad_fp16[i]) / s;
        acc += g * g;
    }
    return acc;
}

/* ---- gradient producer ------------------------------------------------------------------- */

/* G16 (Table II) as it leaves backward when the gradients were accumulated in fp32: one fp32
 * multiplication (e.g. by 1 / accumulation steps), then rounding to binary16 (nearest even,
 * overflow to infinity, gradual underflow).  The paper only names the tensor; producing it from an
 * fp32 accumulator by a scaled cast is a reading.  The flag and norm of the result are those of
 * the functions above applied to the output. */
void lohan_oracle_grad_produce(const float *grad_fp32, uint64_t n, float multiplier,
                               uint16_t *grad_fp16_out)
{
    for (uint64_t i = 0; i < n; ++i) {
        float scaled = grad_fp32[i] * multiplier;
        grad_fp16_out[i] = float_to_half_bits_rne(scaled);
    }
}

/* ---- the step ------------------------------------------------------------------------------ */

typedef struct {
    float inv;    /* fl(1 / loss_scale) */
    float omb1;   /* fl(1 - beta1) */
    float omb2;   /* fl(1 - beta2) */
    float bc1;    /* fp32 rounding of the float64 value 1 - beta1^t */
    float bc2;    /* fp32 rounding of the float64 value 1 - beta2^t */
    float sbc2;   /* fl(sqrt(bc2)) */
    float ss;     /* fl(lr / bc1): bias-corrected step size */
    float decay;  /* fl(1 - fl(lr * wd)): AdamW shrink factor */
} step_scalars;

/* Scalars that do not depend on the element.  t is 1-based: the step being taken. */
static step_scalars make_scalars(float lr, float beta1, float beta2, float wd, int64_t t,
                                 float loss_scale)
{
    step_scalars s;
    s.inv = 1.0f / loss_scale;
    s.omb1 = 1.0f - beta1;
    s.omb2 = 1.0f - beta2;
    s.bc1 = (float)(1.0 - pow((double)beta1, (double)t));
    s.bc2 = (float)(1.0 - pow((double)beta2, (double)t));
    s.sbc2 = sqrtf(s.bc2);
    s.ss = lr / s.bc1;
    float lrwd = lr * wd;
    s.decay = 1.0f - lrwd;
    return s;
}

/* Report the scalars (tests pin them against hand-derived bit patterns). out[8] in the order
 * inv, omb1, omb2, bc1, bc2, sbc2, ss, decay. */
void lohan_oracle_step_scalars(float lr, float beta1, float beta2, float wd, int64_t t,
                               float loss_scale, float *out)
{
    step_scalars s = make_scalars(lr, beta1, beta2, wd, t, loss_scale);
    out[0] = s.inv;  out[1] = s.omb1; out[2] = s.omb2; out[3] = s.bc1;
    out[4] = s.bc2;  out[5] = s.sbc2; out[6] = s.ss;   out[7] = s.decay;
}

/* One element of the update: Kingma & Ba Algorithm 1 with bias correction, eps added to the
 * bias-corrected sqrt(v), and either decoupled decay (AdamW, l2_mode == 0) or the decay folded
 * into the gradient (l2_mode != 0). */
static inline void step_one(float *p, float *m, float *v, uint16_t g16, uint16_t *p16,
                            const step_scalars *s, float beta1, float beta2, float eps, float wd,
                            int l2_mode, int half_out)
{
    float g = half_bits_to_float(g16) * s->inv;        /* unscale */
    if (l2_mode) {
        float wp = wd * (*p);
        g = g + wp;
    }
    float b1m = beta1 * (*m);
    float o1g = s->omb1 * g;
    float m_new = b1m + o1g;                           /* first moment */
    float gg = g * g;
    float b2v = beta2 * (*v);
    float o2gg = s->omb2 * gg;
    float v_new = b2v + o2gg;                          /* second moment */
    float root = sqrtf(v_new);
    float root_hat = root / s->sbc2;                   /* sqrt of the bias-corrected v */
    float den = root_hat + eps;
    float u = m_new / den;
    float pp = l2_mode ? (*p) : (*p) * s->decay;       /* decoupled decay acts on the old p */
    float su = s->ss * u;
    float p_new = pp - su;
    *p = p_new;
    *m = m_new;
    *v = v_new;
    *p16 = half_out ? float_to_half_bits_rne(p_new)    /* 16-bit working copy of the new p */
                    : float_to_bf16_bits_rne(p_new);
}

/* One block step.  Returns the overflow flag (0 or 1); when it is 1 nothing is written.
 * nthreads <= 1 runs the plain serial loop; larger values split the elementwise loop over that
 * many OpenMP threads (the elements are independent, so the result is bit-identical).
 * half_out != 0 emits the 16-bit copy as IEEE binary16 instead of bfloat16. */
int lohan_oracle_adam_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                 const uint16_t *grad_fp16, uint16_t *param_bf16_out, uint64_t n,
                                 float lr, float beta1, float beta2, float eps, float weight_decay,
                                 int64_t step, float loss_scale, int l2_mode, int half_out,
                                 int nthreads)
{
    if (lohan_oracle_grad_overflow_check(grad_fp16, n)) return 1;
    step_scalars s = make_scalars(lr, beta1, beta2, weight_decay, step, loss_scale);
    if (nthreads <= 1) {
        for (uint64_t i = 0; i < n; ++i) {
            step_one(&param_fp32[i], &exp_avg[i], &exp_avg_sq[i], grad_fp16[i],
                     &param_bf16_out[i], &s, beta1, beta2, eps, weight_decay, l2_mode, half_out);
        }
    } else {
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
        for (int64_t i = 0; i < (int64_t)n; ++i) {
            step_one(&param_fp32[i], &exp_avg[i], &exp_avg_sq[i], grad_fp16[i],
                     &param_bf16_out[i], &s, beta1, beta2, eps, weight_decay, l2_mode, half_out);
        }
    }
    return 0;
}

/* Number of threads a parallel call would really get (1 when built without OpenMP). */
int lohan_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Format helpers exposed so tests can pin them against library conversions. */
float lohan_oracle_half_bits_to_float(uint16_t h) { return half_bits_to_float(h); }
uint16_t lohan_oracle_float_to_bf16_bits(float x) { return float_to_bf16_bits_rne(x); }
uint16_t lohan_oracle_float_to_half_bits(float x) { return float_to_half_bits_rne(x); }
