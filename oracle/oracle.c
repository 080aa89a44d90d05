/*
 * CPU oracle for the sharded mixed-precision parameter update (test infrastructure only).
 *
 * This file is the slow, sequential, plain definition that the GPU library is checked against.
 * It is NOT part of the product: only tests, the smoke check and the benchmark's cpu_baseline
 * leg may build, load or call it.  It shares no code with the GPU path.
 *
 * What it computes (paper: Fig. 4a, the Adam parameter-update program; Section 4, "Adam in Data
 * Parallel Training"; Fig. 4b for what lives on one rank's slice):
 *
 *   S_i   = sum over the R incoming fp16 slices of g_r[i]      (the all-reduce with "+")
 *   m'_i  = beta1*m_i + (1-beta1)*S_i
 *   v'_i  = beta2*v_i + (1-beta2)*S_i^2      (the printed program repeats beta1 in this rate;
 *                                             read as the standard second-moment rate)
 *   mhat  = m'/(1-beta1^t),  vhat = v'/(1-beta2^t)
 *   w'_i  = w_i - lr * mhat / sqrt(vhat)     (with the usual epsilon added to the root, and
 *                                             optional weight decay)
 *   the new parameters leave the rank as fp16 (mixed precision, Section 6.1): w16_i.
 *
 * LAMB is cited, not listed, by the paper (Sections 1 and 6.1).  Here it is the published layerwise
 * rule on top of the same moments: u = mhat/(sqrt(vhat)+eps) + wd*w, ratio = ||w|| / ||u|| (1 when
 * either norm is 0), w' = w - lr*ratio*u, with both norms taken over the elements held by this
 * rank (Section 5.2 "Tensor Reduction": each rank reduces locally).
 *
 * Every arithmetic step is in double.  State is kept in fp32 between steps and rounded once,
 * to nearest even, when stored.  Hyper-parameters arrive as the fp32 values the C interface of
 * the GPU library carries and are promoted exactly.
 *
 * Pins (tests/test_oracle_pins.py): exhaustive fp16 decode / sampled encode against numpy's
 * float16, torch.optim.AdamW and torch.optim.Adam in float64 as the R=1 special cases, the
 * first-step closed form lr*g/(|g|+eps), R identical gradients, zero gradients, LAMB closed forms
 * (one-element tensor, pure weight decay, first step with |g| >> eps, ||w|| = 0), scale and
 * permutation invariances, and the bit-level overflow rule.  The general-case LAMB variant
 * (no clamp of the ratio, bias correction on, decay inside the norm) is fixed by this file, not
 * by the paper: beyond those closed forms it is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* ---- fp16 <-> real, written from the IEEE 754 binary16 layout: 1 sign, 5 exponent, 10 fraction ---- */

double oracle_half_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int expo = (h >> 10) & 0x1f;
    const int frac = h & 0x3ff;
    double mag;
    if (expo == 0)       mag = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-24 */
    else if (expo == 31) mag = frac ? (double)NAN : (double)INFINITY;
    else                 mag = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    return sign ? -mag : mag;
}

/* Nearest binary16 to x, ties to even; overflow goes to infinity.  One rounding, straight from the double. */
uint16_t oracle_double_to_half(double x)
{
    const uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
    const double a = fabs(x);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);  /* 65520 is the midpoint above the largest half; the tie goes to the even side, which is infinity */
    if (a < ldexp(1.0, -14)) {
        /* subnormal grid: multiples of 2^-24; 1024 steps lands exactly on the smallest normal */
        const double q = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int ex;
    const double fr = frexp(a, &ex);                 /* a = fr * 2^ex, fr in [0.5, 1) */
    double mant = nearbyint(ldexp(fr, 11));          /* 11 significant bits, in [1024, 2048] */
    int e = ex - 1;                                  /* a = (mant/1024) * 2^e */
    if (mant == 2048.0) { mant = 1024.0; e += 1; }
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)mant - 1024));
}

uint16_t oracle_float_to_half(float x) { return oracle_double_to_half((double)x); }

/* ---- the reduced gradient of one element ---- */

uint16_t oracle_float_to_half(float x);

/* The R slices hold fp16 bit patterns (mixed precision, the paper's main case) or, with grad_f32 == 1, fp32 values
 * (Section 6.1.1 reports Float 32 as qualitatively similar).  grad_f32 == 2 is the unfused baseline as a framework
 * runs it (Section 6.1.1, the AR-Opt schedule over an fp16 all-reduce): fp16 slices whose sum comes back from the
 * reduction as an fp16 tensor, i.e. the fp32 sum rounded to fp16 before the optimizer sees it. */
static double reduced_sum(const void *const *g, int grad_f32, int R, uint64_t i)
{
    double S = 0.0;
    for (int r = 0; r < R; ++r)                                        /* the "+" all-reduce of Fig. 4a */
        S += grad_f32 == 1 ? (double)((const float *)g[r])[i] : oracle_half_to_double(((const uint16_t *)g[r])[i]);
    if (grad_f32 == 2) S = oracle_half_to_double(oracle_float_to_half((float)S));
    return S;
}

/* The overflow decision is taken on the sum as an fp32 value, the precision the GPU path reduces in: fp16 slices
 * cannot overflow it, fp32 slices can. */
static int sum_overflows(double S) { return !isfinite((float)S); }

static double unscale_divisor(float loss_scale, int R, int grad_average)
{
    return (double)loss_scale * (grad_average ? (double)R : 1.0);
}

/* 1 if any reduced gradient of this tensor is inf or NaN, else 0. */
int oracle_grad_overflow(uint64_t n, int R, const void *const *g, int grad_f32)
{
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i)
        if (sum_overflows(reduced_sum(g, grad_f32, R, i))) bad = 1;
    return bad;
}

/* The step was skipped: every output keeps the pre-step value. */
void oracle_keep_tensor(uint64_t n, const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out)
{
    for (uint64_t i = 0; i < n; ++i) {
        w_out[i] = w[i]; m_out[i] = m[i]; v_out[i] = v[i];
        w16_out[i] = oracle_float_to_half(w[i]);
    }
}

/* ---- Adam on one tensor of the slice (Fig. 4a) ----
 * adam_mode 1: decoupled decay, u += wd*w.   adam_mode 0: L2, g += wd*w before the moments.
 * guard_elements != 0: an element whose reduced gradient is not finite keeps its inputs. */
void oracle_adam_tensor(uint64_t n, int R, const void *const *g, int grad_f32,
                        const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out,
                        float lr_f, float beta1_f, float beta2_f, float eps_f, float wd_f,
                        float loss_scale_f, int step, int grad_average, int adam_mode,
                        int guard_elements)
{
    const double lr = lr_f, beta1 = beta1_f, beta2 = beta2_f, eps = eps_f, wd = wd_f;
    const double div = unscale_divisor(loss_scale_f, R, grad_average);
    const double c1 = 1.0 - pow(beta1, (double)step);
    const double c2 = 1.0 - pow(beta2, (double)step);
    for (uint64_t i = 0; i < n; ++i) {
        const double S = reduced_sum(g, grad_f32, R, i);
        if (guard_elements && sum_overflows(S)) {
            w_out[i] = w[i]; m_out[i] = m[i]; v_out[i] = v[i];
            w16_out[i] = oracle_float_to_half(w[i]);
            continue;
        }
        const double wi = w[i];
        double gh = S / div;
        if (adam_mode == 0) gh += wd * wi;
        const double m_ = (double)m[i] * beta1 + (1.0 - beta1) * gh;
        const double v_ = (double)v[i] * beta2 + (1.0 - beta2) * gh * gh;
        const double m1 = m_ / c1;
        const double v1 = v_ / c2;
        double u = m1 / (sqrt(v1) + eps);
        if (adam_mode != 0) u += wd * wi;
        const double p_ = wi - lr * u;
        m_out[i] = (float)m_;
        v_out[i] = (float)v_;
        w_out[i] = (float)p_;
        w16_out[i] = oracle_float_to_half(w_out[i]);
    }
}

/* ---- LAMB on one tensor of the slice ----
 * Returns the two norms through norms[0] = ||w||, norms[1] = ||u|| (may be NULL). */
void oracle_lamb_tensor(uint64_t n, int R, const void *const *g, int grad_f32,
                        const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out,
                        float lr_f, float beta1_f, float beta2_f, float eps_f, float wd_f,
                        float loss_scale_f, int step, int grad_average, double *norms)
{
    const double lr = lr_f, beta1 = beta1_f, beta2 = beta2_f, eps = eps_f, wd = wd_f;
    const double div = unscale_divisor(loss_scale_f, R, grad_average);
    const double c1 = 1.0 - pow(beta1, (double)step);
    const double c2 = 1.0 - pow(beta2, (double)step);
    double sum_w2 = 0.0, sum_u2 = 0.0;
    /* first sweep: moments, and the two sums of squares over this rank's elements */
    for (uint64_t i = 0; i < n; ++i) {
        const double gh = reduced_sum(g, grad_f32, R, i) / div;
        const double wi = w[i];
        const double m_ = (double)m[i] * beta1 + (1.0 - beta1) * gh;
        const double v_ = (double)v[i] * beta2 + (1.0 - beta2) * gh * gh;
        m_out[i] = (float)m_;
        v_out[i] = (float)v_;
        const double u = (m_ / c1) / (sqrt(v_ / c2) + eps) + wd * wi;
        sum_w2 += wi * wi;
        sum_u2 += u * u;
    }
    const double norm_w = sqrt(sum_w2), norm_u = sqrt(sum_u2);
    const double ratio = (norm_w > 0.0 && norm_u > 0.0) ? norm_w / norm_u : 1.0;
    if (norms) { norms[0] = norm_w; norms[1] = norm_u; }
    /* second sweep: the same u, scaled by the tensor's ratio */
    for (uint64_t i = 0; i < n; ++i) {
        const double gh = reduced_sum(g, grad_f32, R, i) / div;
        const double wi = w[i];
        const double m_ = (double)m[i] * beta1 + (1.0 - beta1) * gh;
        const double v_ = (double)v[i] * beta2 + (1.0 - beta2) * gh * gh;
        const double u = (m_ / c1) / (sqrt(v_ / c2) + eps) + wd * wi;
        w_out[i] = (float)(wi - lr * ratio * u);
        w16_out[i] = oracle_float_to_half(w_out[i]);
    }
}
