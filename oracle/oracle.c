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

/* How the R incoming slices are typed, and what type the reduction hands on. */
enum {
    SLICES_F16 = 0,           /* fp16 slices, the sum is handed on in full (mixed precision, the paper's main case)      */
    SLICES_F32 = 1,           /* fp32 slices (Section 6.1.1 evaluates Float 32 elements as well as Float 16)              */
    SLICES_F16_SUM_F16 = 2    /* fp16 slices reduced by an fp16 all-reduce, as a framework's unfused baseline runs it
                                 (Section 6.1.1, the AR-Opt schedule): the optimizer sees the sum as an fp16 tensor       */
};

/* The "+" all-reduce of Fig. 4a, restricted to element i. */
static double reduced_sum(const void *const *slice, int kind, int R, uint64_t i)
{
    double total = 0.0;
    for (int r = 0; r < R; ++r)
        total += kind == SLICES_F32 ? (double)((const float *)slice[r])[i]
                                    : oracle_half_to_double(((const uint16_t *)slice[r])[i]);
    if (kind == SLICES_F16_SUM_F16) total = oracle_half_to_double(oracle_float_to_half((float)total));
    return total;
}

/* The fused reduction works in the largest element type among the tensors of the computation (Section 5.2, "Mixed
 * Precision"), which is fp32 here: fp16 slices are promoted to it, Float 32 slices (Section 6.1.1) have it already,
 * and an all-reduce hands back a tensor of the type it worked in.  The reduced gradient therefore exists as an fp32
 * value and is non-finite exactly when that fp32 value is: an inf/NaN input, infinities of both signs meeting, or a
 * finite sum beyond the fp32 range.  Up to 16 promoted fp16 values cannot leave that range, so for fp16 slices the
 * rule is "some input has all exponent bits set" (which the brute-force pin checks); only fp32 slices can reach the
 * third case. */
static int sum_overflows(double total) { return !isfinite((float)total); }

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

/* ---- the method, per element ----
 * Everything a step needs besides the element's own four numbers, formed once per tensor from the fp32 scalars
 * of the C interface (promoted exactly). */
typedef struct {
    double lr, beta1, beta2, eps, decay;
    double grad_divisor;      /* loss_scale, times R when the slices are averaged instead of summed              */
    double unbias1, unbias2;  /* 1 - beta1^t, 1 - beta2^t with t the 1-based step (the Pow terms of Fig. 4a)    */
    int decay_in_gradient;    /* L2 regularisation: the decay term joins the gradient; otherwise it joins u      */
} step_terms;

static step_terms make_step_terms(float lr, float beta1, float beta2, float eps, float decay, float loss_scale,
                                  int step, int R, int grad_average, int decay_in_gradient)
{
    step_terms k;
    k.lr = lr; k.beta1 = beta1; k.beta2 = beta2; k.eps = eps; k.decay = decay;
    k.grad_divisor = (double)loss_scale * (grad_average ? (double)R : 1.0);
    k.unbias1 = 1.0 - pow(k.beta1, (double)step);
    k.unbias2 = 1.0 - pow(k.beta2, (double)step);
    k.decay_in_gradient = decay_in_gradient;
    return k;
}

/* What one element's reduced gradient does to its moments, and the direction the weight then moves along.
 * (Fig. 4a: exponential averages of the gradient and of its square, each divided by 1 - beta^t, and their
 * quotient.  The second average decays with beta2 and gains with 1 - beta2; epsilon sits outside the root.) */
typedef struct { double first_moment, second_moment, direction; } element_step;

static element_step advance_element(const step_terms *k, double total, double weight, double first_moment,
                                    double second_moment)
{
    element_step e;
    double grad = total / k->grad_divisor;
    if (k->decay_in_gradient) grad += k->decay * weight;
    e.first_moment = k->beta1 * first_moment + (1.0 - k->beta1) * grad;
    e.second_moment = k->beta2 * second_moment + (1.0 - k->beta2) * grad * grad;
    const double mean = e.first_moment / k->unbias1;
    const double spread = sqrt(e.second_moment / k->unbias2);
    e.direction = mean / (spread + k->eps);
    if (!k->decay_in_gradient) e.direction += k->decay * weight;
    return e;
}

/* State is stored as fp32 (one rounding to nearest even), and the fp16 copy is made from the stored fp32 value. */
static void store_weight(double weight_new, float *w_out, uint16_t *w16_out)
{
    *w_out = (float)weight_new;
    *w16_out = oracle_float_to_half(*w_out);
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
    const step_terms k = make_step_terms(lr_f, beta1_f, beta2_f, eps_f, wd_f, loss_scale_f, step, R, grad_average,
                                         adam_mode == 0);
    for (uint64_t i = 0; i < n; ++i) {
        const double total = reduced_sum(g, grad_f32, R, i);
        if (guard_elements && sum_overflows(total)) {
            w_out[i] = w[i]; m_out[i] = m[i]; v_out[i] = v[i];
            w16_out[i] = oracle_float_to_half(w[i]);
            continue;
        }
        const element_step e = advance_element(&k, total, w[i], m[i], v[i]);
        m_out[i] = (float)e.first_moment;
        v_out[i] = (float)e.second_moment;
        store_weight((double)w[i] - k.lr * e.direction, &w_out[i], &w16_out[i]);
    }
}

/* ---- LAMB on one tensor of the slice ----
 * The layerwise rule on top of the same moments: the whole tensor moves along u, scaled by ||w|| / ||u||, both
 * norms over the pre-step weights and the directions of the elements this rank holds; a zero norm gives ratio 1.
 * Returns the two norms through norms[0] = ||w||, norms[1] = ||u|| (may be NULL). */
void oracle_lamb_tensor(uint64_t n, int R, const void *const *g, int grad_f32,
                        const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out,
                        float lr_f, float beta1_f, float beta2_f, float eps_f, float wd_f,
                        float loss_scale_f, int step, int grad_average, double *norms)
{
    const step_terms k = make_step_terms(lr_f, beta1_f, beta2_f, eps_f, wd_f, loss_scale_f, step, R, grad_average, 0);
    double weight_squares = 0.0, direction_squares = 0.0;
    for (uint64_t i = 0; i < n; ++i) {                       /* the norm has to be known before any weight moves */
        const element_step e = advance_element(&k, reduced_sum(g, grad_f32, R, i), w[i], m[i], v[i]);
        m_out[i] = (float)e.first_moment;
        v_out[i] = (float)e.second_moment;
        weight_squares += (double)w[i] * (double)w[i];
        direction_squares += e.direction * e.direction;
    }
    const double weight_norm = sqrt(weight_squares), direction_norm = sqrt(direction_squares);
    const double trust = (weight_norm > 0.0 && direction_norm > 0.0) ? weight_norm / direction_norm : 1.0;
    if (norms) { norms[0] = weight_norm; norms[1] = direction_norm; }
    for (uint64_t i = 0; i < n; ++i) {
        const element_step e = advance_element(&k, reduced_sum(g, grad_f32, R, i), w[i], m[i], v[i]);
        store_weight((double)w[i] - k.lr * trust * e.direction, &w_out[i], &w16_out[i]);
    }
}
