/*
 * CPU oracle for one rank's sharded mixed-precision optimizer step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code with the HIP library and includes none of its headers.
 *
 * Everything here is sequential, one element at a time, double-precision
 * intermediates, one rounding to fp32 at every store.  No SIMD intrinsics, no
 * blocking, no fusion beyond what the definitions state.
 *
 * What the paper fixes (and what it leaves to the standard definitions):
 *   - Experimental settings: bf16 compute copies, fp32 copies of parameters,
 *     gradients and Adam states are kept per rank.
 *   - Adaptive offloading / Motivating example: the optimizer is Adam with a
 *     momentum and a variance buffer; the update runs after backward.
 *   - Fully-sharded approach: parameters are partitioned evenly over ranks
 *     and an all-gather rebuilds them into one large buffer.
 * The paper prints no update formula, so the arithmetic follows the published
 * definitions it cites: Adam (Kingma & Ba, Algorithm 1, epsilon added outside
 * the square root of the bias-corrected second moment), decoupled weight decay
 * (Loshchilov & Hutter), and IEEE-754 round-to-nearest-even for fp32 -> bf16.
 *
 * Pins (tests/test_oracle_*.py): step-1 closed form, zero-gradient pure decay,
 * constant-gradient closed form for bias correction, 50-digit decimal brute
 * force on tiny shards, an independent library AdamW as second opinion,
 * exhaustive bf16 round trip and tie cases, a library bf16 conversion, and
 * brute-force ragged unshard layouts.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { ZCO_ADAMW = 0, ZCO_ADAM_L2 = 1 };

static float zco_bits_to_f32(uint32_t u)
{
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint32_t zco_f32_to_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* bf16 is the upper half of an fp32 word, so widening is exact. */
float zco_bf16_to_f32(uint16_t b)
{
    return zco_bits_to_f32((uint32_t)b << 16);
}

/*
 * fp32 -> bf16, IEEE round-to-nearest, ties to even.  NaN stays NaN (sign and
 * upper payload kept, quiet bit forced); infinities and signed zeros are kept;
 * subnormals are rounded like any other value (no flush); a finite value whose
 * rounding carries out of the exponent becomes infinity, as RNE demands.
 */
uint16_t zco_rne_bf16(float x)
{
    uint32_t bits = zco_f32_to_bits(x);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)((bits >> 16) | 0x0040u);
    uint32_t kept_lsb = (bits >> 16) & 1u;
    bits += 0x7FFFu + kept_lsb;
    return (uint16_t)(bits >> 16);
}

void zco_cast_bf16(const float *src, uint16_t *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = zco_rne_bf16(src[i]);
}

void zco_upcast_bf16(const uint16_t *src, float *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = zco_bf16_to_f32(src[i]);
}

/*
 * One Adam / AdamW step over a flat partition, in place.
 *
 *   t      = step (1-based)
 *   g      = upcast(grad) * grad_scale          (L2 mode: g += wd * p_old)
 *   m      = beta1 * m + (1 - beta1) * g        -> stored as fp32
 *   v      = beta2 * v + (1 - beta2) * g * g    -> stored as fp32
 *   m_hat  = m / (1 - beta1^t),  v_hat = v / (1 - beta2^t)   (stored m, v)
 *   p      = p_old * (1 - lr * wd)  [AdamW only]  -  lr * m_hat / (sqrt(v_hat) + eps)
 *   bf16_out = RNE(p) taken from the stored fp32 p, when requested
 *
 * Hyper-parameters arrive as fp32 values (that is what the boundary carries)
 * and are widened to double before use.  If skip != 0 nothing is touched
 * (loss-scaling convention: an overflowed step is dropped).
 */
void zco_adam_step(float *p, float *m, float *v, const void *g, int g_is_bf16,
                   int64_t n, float lr_f, float beta1_f, float beta2_f,
                   float eps_f, float wd_f, float grad_scale_f, int64_t step,
                   int mode, uint16_t *bf16_out, int skip)
{
    if (skip)
        return;
    const double lr = lr_f, beta1 = beta1_f, beta2 = beta2_f, eps = eps_f;
    const double wd = wd_f, grad_scale = grad_scale_f;
    const double bc1 = 1.0 - pow(beta1, (double)step);
    const double bc2 = 1.0 - pow(beta2, (double)step);
    const float *g32 = (const float *)g;
    const uint16_t *g16 = (const uint16_t *)g;

    for (int64_t i = 0; i < n; ++i) {
        double gi = g_is_bf16 ? (double)zco_bf16_to_f32(g16[i]) : (double)g32[i];
        gi *= grad_scale;
        const double p_old = (double)p[i];
        if (mode == ZCO_ADAM_L2)
            gi += wd * p_old;

        const double m_new = beta1 * (double)m[i] + (1.0 - beta1) * gi;
        const double v_new = beta2 * (double)v[i] + (1.0 - beta2) * gi * gi;
        m[i] = (float)m_new;
        v[i] = (float)v_new;

        const double m_hat = (double)m[i] / bc1;
        const double v_hat = (double)v[i] / bc2;
        double p_dec = p_old;
        if (mode == ZCO_ADAMW)
            p_dec = p_old * (1.0 - lr * wd);
        p[i] = (float)(p_dec - lr * m_hat / (sqrt(v_hat) + eps));

        if (bf16_out)
            bf16_out[i] = zco_rne_bf16(p[i]);
    }
}

/*
 * The same step with every per-element intermediate in fp32 (each operation rounded to
 * fp32, no fused multiply-add; built with contraction off).  A second opinion that tells
 * "rounding" from "formula" when a kernel disagrees with zco_adam_step: a kernel that
 * computes in fp32 should sit within a few ulp of this one, a wrong formula sits far from
 * both.  The once-per-call scalars (bias corrections, 1 - lr*wd is not formed: the decay is
 * taken as p - (lr*wd)*p) are computed in double and rounded to fp32 once.
 * Pinned by staying within a few fp32 ulp of zco_adam_step and by the step-1 closed form.
 */
void zco_adam_step_f32(float *p, float *m, float *v, const void *g, int g_is_bf16,
                       int64_t n, float lr_f, float beta1_f, float beta2_f,
                       float eps_f, float wd_f, float grad_scale_f, int64_t step,
                       int mode, uint16_t *bf16_out, int skip)
{
    if (skip != 0)
        return;
    const double bc1 = 1.0 - pow((double)beta1_f, (double)step);
    const double bc2 = 1.0 - pow((double)beta2_f, (double)step);
    const float step_size = (float)((double)lr_f / bc1);
    const float inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
    const float one_minus_beta1 = (float)(1.0 - (double)beta1_f);
    const float one_minus_beta2 = (float)(1.0 - (double)beta2_f);
    const float lr_wd = (float)((double)lr_f * (double)wd_f);
    const float *g32 = (const float *)g;
    const uint16_t *g16 = (const uint16_t *)g;

    for (int64_t i = 0; i < n; ++i) {
        float gi = g_is_bf16 ? zco_bf16_to_f32(g16[i]) : g32[i];
        gi = gi * grad_scale_f;
        const float p_old = p[i];
        if (mode == ZCO_ADAM_L2)
            gi = gi + wd_f * p_old;

        const float m_a = beta1_f * m[i];
        const float m_b = one_minus_beta1 * gi;
        m[i] = m_a + m_b;
        const float v_a = beta2_f * v[i];
        const float v_b = one_minus_beta2 * gi;
        const float v_c = v_b * gi;
        v[i] = v_a + v_c;

        const float root = sqrtf(v[i]);
        const float denom_a = root * inv_sqrt_bc2;
        const float denom = denom_a + eps_f;
        const float ratio = m[i] / denom;
        const float delta = step_size * ratio;
        float p_dec = p_old;
        if (mode == ZCO_ADAMW) {
            const float shrink = lr_wd * p_old;
            p_dec = p_old - shrink;
        }
        const float p_new = p_dec - delta;
        p[i] = p_new;

        if (bf16_out)
            bf16_out[i] = zco_rne_bf16(p_new);   /* p_new is the stored fp32 value */
    }
}

/*
 * Sum of squares of the (upcast) gradient in double, and a flag that is 1
 * when any element is NaN or infinite.  The sum skips nothing: a non-finite
 * element makes the sum non-finite as IEEE says.
 */
void zco_grad_sqnorm(const void *g, int g_is_bf16, int64_t n, double *sqnorm,
                     int32_t *found_inf)
{
    const float *g32 = (const float *)g;
    const uint16_t *g16 = (const uint16_t *)g;
    double acc = 0.0;
    int32_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        const double gi = g_is_bf16 ? (double)zco_bf16_to_f32(g16[i]) : (double)g32[i];
        if (!isfinite(gi))
            bad = 1;
        acc += gi * gi;
    }
    *sqnorm = acc;
    *found_inf = bad;
}

/*
 * Unshard copy: for every segment s, dst_s[j] = gathered[src_offset[s] + j],
 * j in [0, numel[s]).  A bit copy of 16-bit words.
 */
void zco_unshard(const uint16_t *gathered, const int64_t *src_offset,
                 uint16_t *const *dst, const int64_t *numel, int64_t nsegs)
{
    for (int64_t s = 0; s < nsegs; ++s)
        for (int64_t j = 0; j < numel[s]; ++j)
            dst[s][j] = gathered[src_offset[s] + j];
}

/*
 * Gradient accumulation into the fp32 gradient partition (the paper keeps fp32
 * gradients, Experimental settings, and accumulates several forward/backward
 * passes before one update, Selective unsharding):
 *   acc[i] = acc[i] + upcast(micro[i]) * scale, one rounding to fp32 per store.
 */
void zco_grad_accumulate(float *acc, const void *micro, int micro_is_bf16, int64_t n, float scale_f)
{
    const double scale = scale_f;
    const float *g32 = (const float *)micro;
    const uint16_t *g16 = (const uint16_t *)micro;
    for (int64_t i = 0; i < n; ++i) {
        const double gi = micro_is_bf16 ? (double)zco_bf16_to_f32(g16[i]) : (double)g32[i];
        acc[i] = (float)((double)acc[i] + gi * scale);
    }
}

/*
 * Gradient-clipping coefficient with loss-scale removal (the usual mixed-precision
 * recipe; not in the paper): norm = sqrt(sqnorm) * inv_loss_scale,
 * scale = inv_loss_scale * min(1, max_norm / (norm + 1e-6)); max_norm = 0 means no
 * clipping.  Double arithmetic, one rounding to fp32.
 */
float zco_clip_scale(float sqnorm, float max_norm, float inv_loss_scale)
{
    const double norm = sqrt((double)sqnorm) * (double)inv_loss_scale;
    double coef = 1.0;
    if (max_norm > 0.0f) {
        coef = (double)max_norm / (norm + 1e-6);
        if (coef > 1.0)
            coef = 1.0;
    }
    return (float)((double)inv_loss_scale * coef);
}
