/*
 * CPU oracle for the model-parallel epilogue (test infrastructure only; shares no code with the GPU path).
 *
 * Paper, Fig. 3 (the running example: the end of a model-parallel self-attention / MLP block) after the
 * schedule of Fig. 5 program 3 (split the all-reduce, reorder the all-gather behind the pointwise work, fuse):
 * on one rank's slice of the [B*S, H] output,
 *
 *     sum_i = partial_0[i] + ... + partial_{R-1}[i]        (the "+" all-reduce of the local MatMul results)
 *     out_i = Dropout(sum_i + b[col(i)], p) + r_i           (bias is replicated and broadcast along H)
 *
 * all tensors fp16.  Dropout keeps an element with probability 1 - p and scales kept values by 1/(1-p).  The
 * paper does not say how the random mask is drawn; here it is a counter-based generator so that the mask depends
 * only on (seed, global element index) and both sides can reproduce it: Philox4x32-10 (Salmon, Moraes, Dror,
 * Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11) with counter = (index/4 low, index/4 high, 0, 0),
 * key = (seed low, seed high); element `index` takes output word index%4 and is kept iff word >= floor(p*2^32).
 * Arithmetic in double, one rounding to fp16 at the end.
 *
 * Pins (tests/test_oracle_epilogue.py): the generator's published known-answer vectors, numpy for p = 0, dropped
 * elements equal the residual bit for bit, kept fraction, slice and rank-order invariance.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

double oracle_half_to_double(uint16_t h);
uint16_t oracle_double_to_half(double x);

/* One Philox4x32 block with 10 rounds. */
void oracle_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;          /* round multipliers */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;          /* key schedule increments (Weyl sequence) */
    uint32_t c[4] = {ctr_in[0], ctr_in[1], ctr_in[2], ctr_in[3]};
    uint32_t k[2] = {key_in[0], key_in[1]};
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k[0] += W0; k[1] += W1; }
        const uint64_t p0 = M0 * (uint64_t)c[0], p1 = M1 * (uint64_t)c[2];
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c[1] ^ k[0], n1 = lo1, n2 = hi0 ^ c[3] ^ k[1], n3 = lo0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* The 32 random bits that decide element `index` of the full tensor. */
uint32_t oracle_dropout_word(uint64_t seed, uint64_t index)
{
    const uint64_t block = index / 4;
    const uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), 0u, 0u};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    oracle_philox4x32_10(ctr, key, w);
    return w[index % 4];
}

/* threshold below which an element is dropped: floor(p * 2^32) */
uint32_t oracle_dropout_threshold(float p) { return (uint32_t)floor((double)p * 4294967296.0); }

/*
 * out[i] for i in [0, n): element i of this rank's slice is element first + i of the full tensor.
 * kept (optional, n bytes) receives the mask.
 */
void oracle_mp_epilogue(uint64_t n, uint64_t first, uint32_t hidden, int R, const uint16_t *const *partial,
                        const uint16_t *bias, const uint16_t *residual, uint16_t *out,
                        float p_f, uint64_t seed, uint8_t *kept)
{
    const double scale = 1.0 / (1.0 - (double)p_f);
    const uint32_t threshold = oracle_dropout_threshold(p_f);
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t gi = first + i;
        double sum = 0.0;
        for (int r = 0; r < R; ++r) sum += oracle_half_to_double(partial[r][i]);
        const double x = sum + oracle_half_to_double(bias[gi % hidden]);
        const int keep = oracle_dropout_word(seed, gi) >= threshold;
        const double d = keep ? x * scale : 0.0;
        out[i] = oracle_double_to_half(d + oracle_half_to_double(residual[i]));
        if (kept) kept[i] = (uint8_t)keep;
    }
}
