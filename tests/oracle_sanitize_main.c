/* Host-only driver for the sanitizer leg of the test suite: calls every routine of oracle/oracle.c and
 * oracle/epilogue.c over inputs that reach their corners (every fp16 bit pattern, inf/NaN, empty tensors, 16
 * slices, fp32 slices, the fp16 intermediate, guard and skip paths, slices that start deep inside the tensor).
 * Built with -fsanitize=address,undefined -fno-sanitize-recover=all, so any out-of-bounds access, misaligned
 * access, signed overflow or invalid shift ends the program with a non-zero status.  Prints a checksum of all
 * outputs, which tests/test_oracle_sanitizers.py compares with the same program built without sanitizers. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double oracle_half_to_double(uint16_t h);
uint16_t oracle_double_to_half(double x);
uint16_t oracle_float_to_half(float x);
int oracle_grad_overflow(uint64_t n, int R, const void *const *g, int grad_f32);
void oracle_keep_tensor(uint64_t n, const float *w, const float *m, const float *v, float *w_out, float *m_out, float *v_out,
                        uint16_t *w16_out);
void oracle_adam_tensor(uint64_t n, int R, const void *const *g, int grad_f32, const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out, float lr, float beta1, float beta2,
                        float eps, float wd, float loss_scale, int step, int grad_average, int adam_mode, int guard_elements);
void oracle_lamb_tensor(uint64_t n, int R, const void *const *g, int grad_f32, const float *w, const float *m, const float *v,
                        float *w_out, float *m_out, float *v_out, uint16_t *w16_out, float lr, float beta1, float beta2,
                        float eps, float wd, float loss_scale, int step, int grad_average, double *norms);
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t oracle_dropout_word(uint64_t seed, uint64_t index);
uint32_t oracle_dropout_threshold(float p);
void oracle_mp_epilogue(uint64_t n, uint64_t first, uint32_t hidden, int R, const uint16_t *const *partial, const uint16_t *bias,
                        const uint16_t *residual, uint16_t *out, float p, uint64_t seed, uint8_t *kept);

static uint64_t sum = 1469598103934665603ull;
static void mix(const void *p, size_t bytes)
{
    const unsigned char *b = (const unsigned char *)p;
    for (size_t i = 0; i < bytes; ++i) sum = (sum ^ b[i]) * 1099511628211ull;
}
static uint64_t rng = 88172645463325252ull;
static uint64_t next(void) { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; }
static float unit(void) { return (float)((double)(next() >> 11) / 9007199254740992.0 * 2.0 - 1.0); }

#define MAXR 16
static void optimizer_case(uint64_t n, int R, int kind, int plant)
{
    /* exact-size heap blocks, so that an access one element past the end is caught */
    float *w = malloc(n * 4 + 1), *m = malloc(n * 4 + 1), *v = malloc(n * 4 + 1);
    float *wo = malloc(n * 4 + 1), *mo = malloc(n * 4 + 1), *vo = malloc(n * 4 + 1);
    uint16_t *h = malloc(n * 2 + 1);
    void *g[MAXR];
    const void *gc[MAXR];
    for (uint64_t i = 0; i < n; ++i) { w[i] = 0.02f * unit(); m[i] = 3e-3f * unit(); v[i] = 1e-6f * unit() * unit() + 0.f; if (v[i] < 0) v[i] = -v[i]; }
    for (int r = 0; r < R; ++r) {
        g[r] = malloc(n * (kind == 1 ? 4 : 2) + 1);
        for (uint64_t i = 0; i < n; ++i) {
            if (kind == 1) ((float *)g[r])[i] = 1e-2f * unit();
            else ((uint16_t *)g[r])[i] = oracle_float_to_half(1e-2f * unit());
        }
        gc[r] = g[r];
    }
    if (plant && n > 0) {
        if (kind == 1) { ((float *)g[0])[n / 2] = INFINITY; ((float *)g[R - 1])[n - 1] = 3e38f; ((float *)g[0])[n - 1] = 3e38f; }
        else { ((uint16_t *)g[0])[n / 2] = 0x7C00; ((uint16_t *)g[R - 1])[0] = 0x7E01; ((uint16_t *)g[R - 1])[n - 1] = 0x7BFF; }
    }
    const int flag = oracle_grad_overflow(n, R, gc, kind);
    mix(&flag, sizeof flag);
    for (int mode = 0; mode < 2; ++mode)
        for (int guard = 0; guard < 2; ++guard) {
            oracle_adam_tensor(n, R, gc, kind, w, m, v, wo, mo, vo, h, 1e-3f, 0.9f, 0.999f, 1e-6f, 0.01f, kind == 0 ? 8.f : 1.f,
                               1 + mode * 6, guard, mode, guard);
            mix(wo, n * 4); mix(mo, n * 4); mix(vo, n * 4); mix(h, n * 2);
        }
    if (kind != 2) {
        double norms[2] = {0, 0};
        oracle_lamb_tensor(n, R, gc, kind, w, m, v, wo, mo, vo, h, 1e-3f, 0.9f, 0.999f, 1e-6f, 0.01f, 1.f, 2, 0, norms);
        oracle_lamb_tensor(n, R, gc, kind, w, m, v, wo, mo, vo, h, 1e-3f, 0.f, 0.f, 0.f, 0.f, 1.f, 1, 1, NULL);
        if (!plant) { mix(wo, n * 4); mix(h, n * 2); mix(norms, sizeof norms); }      /* NaN payloads are not compared */
    }
    oracle_keep_tensor(n, w, m, v, wo, mo, vo, h);
    mix(wo, n * 4); mix(h, n * 2);
    for (int r = 0; r < R; ++r) free(g[r]);
    free(w); free(m); free(v); free(wo); free(mo); free(vo); free(h);
}

static void epilogue_case(uint64_t n, uint64_t first, uint32_t hidden, int R, float p)
{
    uint16_t *part[MAXR];
    const uint16_t *pc[MAXR];
    for (int r = 0; r < R; ++r) {
        part[r] = malloc(n * 2 + 1);
        for (uint64_t i = 0; i < n; ++i) part[r][i] = oracle_float_to_half(0.5f * unit());
        pc[r] = part[r];
    }
    uint16_t *bias = malloc(hidden * 2 + 1), *res = malloc(n * 2 + 1), *out = malloc(n * 2 + 1);
    uint8_t *kept = malloc(n + 1);
    for (uint32_t i = 0; i < hidden; ++i) bias[i] = oracle_float_to_half(0.1f * unit());
    for (uint64_t i = 0; i < n; ++i) res[i] = oracle_float_to_half(unit());
    if (n > 2) { res[1] = 0x7C00; part[0][2] = 0xFC00; }
    oracle_mp_epilogue(n, first, hidden, R, pc, bias, res, out, p, 0x123456789abcdefull, kept);
    oracle_mp_epilogue(n, first, hidden, R, pc, bias, res, out, p, 7, NULL);
    mix(out, n * 2); mix(kept, n);
    for (int r = 0; r < R; ++r) free(part[r]);
    free(bias); free(res); free(out); free(kept);
}

int main(void)
{
    for (uint32_t b = 0; b < 65536; ++b) {
        const double d = oracle_half_to_double((uint16_t)b);
        const uint16_t back = oracle_double_to_half(d);
        mix(&back, 2);
    }
    const double edges[] = {0.0, -0.0, 65504.0, 65519.999, 65520.0, 1e300, -1e300, 5e-324, 2.9802322387695312e-08, 6.103515625e-05,
                            INFINITY, -INFINITY, NAN};
    for (size_t i = 0; i < sizeof edges / sizeof edges[0]; ++i) {
        const uint16_t a = oracle_double_to_half(edges[i]), b = oracle_float_to_half((float)edges[i]);
        if (edges[i] == edges[i]) { mix(&a, 2); mix(&b, 2); }
    }
    const uint64_t sizes[] = {0, 1, 2, 7, 1000, 4097};
    for (size_t s = 0; s < sizeof sizes / sizeof sizes[0]; ++s)
        for (int kind = 0; kind < 3; ++kind) {
            optimizer_case(sizes[s], 1, kind, 0);
            optimizer_case(sizes[s], 16, kind, 0);
            optimizer_case(sizes[s], 5, kind, 1);
        }
    uint32_t ctr[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}, key[2] = {0xffffffffu, 0xffffffffu}, out[4];
    oracle_philox4x32_10(ctr, key, out);
    mix(out, sizeof out);
    const uint32_t w0 = oracle_dropout_word(~0ull, ~0ull), t0 = oracle_dropout_threshold(0.f), t1 = oracle_dropout_threshold(0.99999994f);
    mix(&w0, 4); mix(&t0, 4); mix(&t1, 4);
    epilogue_case(0, 0, 8, 1, 0.1f);
    epilogue_case(1, 0xfffffffffffffff0ull, 8, 16, 0.5f);
    epilogue_case(5000, 3072ull * 1000003ull + 8, 3072, 8, 0.1f);
    epilogue_case(777, 96 * 5, 96, 3, 0.f);
    printf("%016llx\n", (unsigned long long)sum);
    return 0;
}
