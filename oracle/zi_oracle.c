/*
 * zi_oracle — plain, slow, single-threaded CPU reference for the mixed-precision
 * optimizer step.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
 * call, link or import it.  It shares no code with the HIP library.
 *
 * What it computes, and where the paper fixes it:
 *   - which arrays exist and their precision: low-precision parameters and
 *     gradients, fp32 momentum, variance and master parameters (Section 3,
 *     "Memory for Model States"); parameter updates are done in fp32
 *     (Section 2, "Adam Optimizer and Mixed Precision Training");
 *   - the step reads every state once and writes it once (Section 4.1,
 *     "AIT w.r.t. Optimizer States") and is independent per element
 *     (Section 5.2.2), so one flat loop over the owned partition is the whole
 *     definition (Section 2, "ZeRO": each rank updates only what it owns).
 * The paper cites Adam and mixed-precision training without writing their
 * equations, a loss-scale rule, an overflow rule, clipping or a rounding mode.
 * This file takes the standard published definitions: bias-corrected Adam with
 * decoupled weight decay (AdamW), eps added outside the square root, dynamic
 * loss scaling's skip-on-overflow rule, global-L2-norm clipping with
 * clip = max_norm / (norm + 1e-6), and round-to-nearest-even casts.
 *
 * Precision: every per-element operation is IEEE-754 binary32, round to
 * nearest even, in the order written below, with fused multiply-adds only
 * where fmaf() is written (compile with -ffp-contract=off).  Every per-step
 * scalar and the sum of squares are computed in double.
 *
 * Pins (see tests/): closed form of the first step, invariants, a textbook
 * double-precision evaluation on small inputs, exhaustive cast checks against
 * the CPU's hardware converter and against a compare-neighbours formulation,
 * closed-form norms, printed bias-correction constants.
 */
#include "zi_oracle.h"

#include <math.h>
#include <string.h>

/* ------------------------------------------------------------------ casts */

static inline uint32_t f32_bits(float x) { uint32_t b; memcpy(&b, &x, 4); return b; }
static inline float bits_f32(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }

/* Low-precision -> fp32, exact (Section 3: parameters and gradients are kept in 16-bit formats). */
float zio_bf16_to_f32(uint16_t h)
{
    return bits_f32((uint32_t)h << 16);
}

float zio_f16_to_f32(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1Fu;
    const uint32_t f = h & 0x3FFu;
    if (e == 0x1Fu) return bits_f32(sign | 0x7F800000u | (f << 13));   /* inf, NaN */
    if (e == 0) {                                                      /* zero, subnormal: f * 2^-24 */
        float mag = ldexpf((float)f, -24);
        return sign ? -mag : mag;
    }
    return bits_f32(sign | ((e + 112u) << 23) | (f << 13));
}

/* fp32 -> bf16, round to nearest, ties to even; NaN stays NaN (quieted).  The low-precision copy of
 * the updated fp32 parameter (Section 3; Table 1's "fp16 param" placement); the paper names no rounding
 * mode, IEEE-754 round-to-nearest-even is the reading taken. */
uint16_t zio_f32_to_bf16(float x)
{
    uint32_t b = f32_bits(x);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x0040u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

/* fp32 -> fp16, round to nearest, ties to even; subnormals kept; overflow -> inf (same passage). */
uint16_t zio_f32_to_f16(float x)
{
    const uint32_t b = f32_bits(x);
    const uint16_t sign = (uint16_t)((b >> 16) & 0x8000u);
    const uint32_t a = b & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((a >> 13) & 0x3FFu));
    if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);  /* >= 65520: rounds to inf (or is inf) */
    if (a < 0x38800000u) {                                    /* below 2^-14: fp16 subnormal or zero */
        const uint32_t e = a >> 23;
        if (e < 102u) return sign;                            /* below 2^-25: rounds to zero */
        const uint32_t m = (a & 0x7FFFFFu) | 0x800000u;       /* value = m * 2^(e-150) = m * 2^(e-126) * 2^-24 */
        const uint32_t shift = 126u - e;                      /* 14..24 */
        uint32_t h = m >> shift;
        const uint32_t rem = m & ((1u << shift) - 1u);
        const uint32_t half = 1u << (shift - 1u);
        if (rem > half || (rem == half && (h & 1u))) ++h;
        return (uint16_t)(sign | h);
    }
    uint32_t h = (a - 0x38000000u) >> 13;
    const uint32_t rem = a & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;
    return (uint16_t)(sign | h);
}

static inline float widen(uint16_t h, int dtype)
{
    return dtype == ZIO_BF16 ? zio_bf16_to_f32(h) : zio_f16_to_f32(h);
}

static inline uint16_t narrow(float x, int dtype)
{
    return dtype == ZIO_BF16 ? zio_f32_to_bf16(x) : zio_f32_to_f16(x);
}

void zio_cast_array(const float* x, uint16_t* out, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; ++i) out[i] = narrow(x[i], dtype);
}

void zio_widen_array(const uint16_t* x, float* out, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; ++i) out[i] = widen(x[i], dtype);
}

/* ------------------------------------------------ gradient norm and overflow */

/* Global gradient norm and overflow flag: not written down in the paper (Section 2 only cites
 * mixed-precision training); the standard dynamic-loss-scaling rule is taken. */
void zio_sumsq_init(zio_sumsq_state* st)
{
    st->sum = 0.0;
    st->comp = 0.0;
    st->found_inf = 0;
}

/*
 * Adds the squares of one gradient tensor, in index order, to a compensated
 * (Neumaier) double sum.  Each square is exact in double for bf16 and fp16
 * inputs.  found_inf is raised by any element whose exponent field is all ones
 * (+-inf or any NaN), tested on the raw 16-bit pattern.
 */
void zio_sumsq_accumulate(zio_sumsq_state* st, const uint16_t* g, int64_t n, int dtype)
{
    const uint16_t expmask = dtype == ZIO_BF16 ? 0x7F80u : 0x7C00u;
    double sum = st->sum, comp = st->comp;
    for (int64_t i = 0; i < n; ++i) {
        if ((g[i] & expmask) == expmask) { st->found_inf = 1; continue; }
        const double x = (double)widen(g[i], dtype);
        const double sq = x * x;
        const double t = sum + sq;
        if (fabs(sum) >= fabs(sq)) comp += (sum - t) + sq;
        else                       comp += (sq - t) + sum;
        sum = t;
    }
    st->sum = sum;
    st->comp = comp;
}

double zio_sumsq_value(const zio_sumsq_state* st)
{
    return st->sum + st->comp;
}

/* ------------------------------------------------------ per-step scalars */

/*
 * All in double, each constant rounded once to fp32 where the element loop
 * uses it.  step is the 1-based index of the step being taken.
 *   bias corrections  bc1 = 1 - beta1^step,  bc2 = 1 - beta2^step
 *   step_size = lr / bc1;  the denominator is sqrt(v)/sqrt(bc2) + eps
 *   norm = sqrt(sumsq) / loss_scale   (global L2 norm of the unscaled gradients)
 *   clip = max_norm / (norm + 1e-6) when that is below 1, else 1
 *   gscale = clip / loss_scale        (the factor applied to each raw gradient)
 */
int zio_scalars(const zio_config* c, int have_norm, double sumsq, zio_scalars_out* o)
{
    if (!c || !o) return -1;
    if (c->step < 1 || !(c->loss_scale > 0.0f) || isinf(c->loss_scale)) return -1;
    if (!(c->beta1 >= 0.0f && c->beta1 < 1.0f) || !(c->beta2 >= 0.0f && c->beta2 < 1.0f)) return -1;
    if (!(c->eps >= 0.0f)) return -1;
    if (c->mode != ZIO_MODE_ADAMW && c->mode != ZIO_MODE_ADAM_L2) return -1;
    const double b1 = (double)c->beta1, b2 = (double)c->beta2;
    o->omb1 = (float)(1.0 - b1);
    o->omb2 = (float)(1.0 - b2);
    o->bc1 = 1.0 - pow(b1, (double)c->step);
    o->bc2 = 1.0 - pow(b2, (double)c->step);
    o->step_size = (float)((double)c->lr / o->bc1);
    o->inv_sqrt_bc2 = (float)(1.0 / sqrt(o->bc2));
    o->decay = c->mode == ZIO_MODE_ADAMW ? (float)((double)c->lr * (double)c->weight_decay) : 0.0f;
    const double ls = (double)c->loss_scale;
    double clip = 1.0;
    o->norm = 0.0;
    if (have_norm) {
        o->norm = sqrt(sumsq) / ls;
        if (c->max_grad_norm > 0.0f && o->norm + 1e-6 > (double)c->max_grad_norm)
            clip = (double)c->max_grad_norm / (o->norm + 1e-6);
    }
    o->clip = clip;
    o->gscale = (float)(clip / ls);
    return 0;
}

/* ------------------------------------------------------------- the update */

/*
 * One AdamW (or Adam with L2 regularisation) step over n elements, in place.
 * found_inf != 0 means the step is skipped: nothing is written.
 *
 * Real-number meaning (AdamW): with g the unscaled, clipped gradient,
 *   m' = b1 m + (1-b1) g,  v' = b2 v + (1-b2) g^2,
 *   p' = p (1 - lr wd) - lr (m'/bc1) / (sqrt(v'/bc2) + eps),
 *   p_lp = round_to_nearest_even(p').
 */
int zio_adamw(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, int64_t n, int dtype,
              const zio_config* c, int have_norm, double sumsq, int found_inf)
{
    zio_scalars_out s;
    if (n < 0 || (dtype != ZIO_BF16 && dtype != ZIO_FP16)) return -1;
    if (zio_scalars(c, have_norm, sumsq, &s) != 0) return -1;
    if (found_inf) return 1;

    const float beta1 = c->beta1, beta2 = c->beta2, eps = c->eps, wd = c->weight_decay;
    const int l2 = c->mode == ZIO_MODE_ADAM_L2;

    for (int64_t i = 0; i < n; ++i) {
        float gi = widen(g[i], dtype);                 /* exact */
        gi = gi * s.gscale;                            /* unscale and clip */
        if (l2) gi = fmaf(wd, p[i], gi);               /* L2 mode: decay enters the gradient */
        const float m1 = fmaf(beta1, m[i], s.omb1 * gi);
        const float v1 = fmaf(beta2, v[i], s.omb2 * (gi * gi));
        const float d = fmaf(sqrtf(v1), s.inv_sqrt_bc2, eps);
        const float q = m1 / d;
        const float pd = fmaf(-s.decay, p[i], p[i]);   /* decoupled decay on the old parameter */
        const float p1 = fmaf(-s.step_size, q, pd);
        m[i] = m1;
        v[i] = v1;
        p[i] = p1;
        if (p_lp) p_lp[i] = narrow(p1, dtype);
    }
    return 0;
}

int zio_cpu_ok(void)
{
    return __builtin_cpu_supports("fma") ? 1 : 0;
}
