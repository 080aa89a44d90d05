"""Pins of the epilogue oracle (paper, Fig. 3: out = Dropout(AllReduce(layer) + b, p) + r on one rank's slice)."""
import os

import numpy as np
import pytest

import oracle
from util import bits_to_f64, half_bits

HERE = os.path.dirname(os.path.abspath(__file__))


def kat_vectors():
    out = []
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out.append((w[:4], w[4:6], tuple(w[6:])))
    return out


def test_philox_known_answers():
    vs = kat_vectors()
    assert len(vs) == 3
    for ctr, key, want in vs:
        assert oracle.philox4x32_10(ctr, key) == want


def test_dropout_word_is_the_block_word_of_the_global_index():
    seed = 0x0123456789ABCDEF
    for index in (0, 1, 2, 3, 4, 7, 1023, 2 ** 32 + 5, 2 ** 40 + 3):
        block = index // 4
        words = oracle.philox4x32_10([block & 0xFFFFFFFF, block >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.dropout_word(seed, index) == words[index % 4]
    assert oracle.dropout_threshold(0.0) == 0
    assert oracle.dropout_threshold(0.5) == 2 ** 31
    assert oracle.dropout_threshold(float(np.float32(0.1))) == int(np.floor(float(np.float32(0.1)) * 2 ** 32))


def test_double_to_half_rounds_once():
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.normal(0, s, 3000) for s in (1e-7, 1e-4, 1, 1e3)] + [np.array([65519.999, 65520.0, 2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -30)])])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)              # numpy rounds double -> half in one step
    got = np.array([oracle.double_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
    # a value where rounding through fp32 first would go the other way: just above a half-way point of fp16
    x = 1.0 + 2.0 ** -11 + 2.0 ** -40
    assert oracle.double_to_half(x) == 0x3C01 and np.float16(np.float32(x)).view(np.uint16) == 0x3C00


def make_case(rng, n, R, hidden, scale=0.5):
    partials = [half_bits(rng.normal(0, scale, n)) for _ in range(R)]
    bias = half_bits(rng.normal(0, 0.1, hidden))
    residual = half_bits(rng.normal(0, 1.0, n))
    return partials, bias, residual


def test_no_dropout_is_sum_plus_bias_plus_residual():
    rng = np.random.default_rng(1)
    n, R, H, first = 5000, 8, 96, 960
    partials, bias, residual = make_case(rng, n, R, H)
    out, kept = oracle.mp_epilogue(partials, bias, residual, first, 0.0, 7)
    assert kept.all()
    total = sum(bits_to_f64(x) for x in partials) + bits_to_f64(bias)[(first + np.arange(n)) % H] + bits_to_f64(residual)
    assert np.array_equal(out, total.astype(np.float16).view(np.uint16))


def test_dropout_mask_scale_and_residual():
    rng = np.random.default_rng(2)
    n, R, H, first, p, seed = 40000, 4, 128, 256, 0.1, 99
    partials, bias, residual = make_case(rng, n, R, H)
    out, kept = oracle.mp_epilogue(partials, bias, residual, first, p, seed)
    pf = float(np.float32(p))
    thr = oracle.dropout_threshold(pf)
    brute = np.array([oracle.dropout_word(seed, first + i) >= thr for i in range(0, n, 37)])
    assert np.array_equal(kept[::37].astype(bool), brute)
    frac = kept.mean()
    assert abs(frac - (1 - pf)) < 4 * np.sqrt(pf * (1 - pf) / n)                  # binomial, 4 sigma
    dropped = kept == 0
    assert np.array_equal(out[dropped], residual[dropped])                          # 0 + r rounds to r exactly
    x = sum(bits_to_f64(a) for a in partials) + bits_to_f64(bias)[(first + np.arange(n)) % H]
    want = (x / (1 - pf) + bits_to_f64(residual)).astype(np.float16).view(np.uint16)
    assert np.array_equal(out[~dropped], want[~dropped])
    # a different seed gives a different mask; the same seed the same one
    _, kept2 = oracle.mp_epilogue(partials, bias, residual, first, p, seed + 1)
    assert (kept2 != kept).mean() > 0.1
    _, kept3 = oracle.mp_epilogue(partials, bias, residual, first, p, seed)
    assert np.array_equal(kept3, kept)


def test_slices_compose_and_rank_order_is_irrelevant():
    rng = np.random.default_rng(3)
    n, R, H, p, seed = 6000, 8, 48, 0.25, 5
    partials, bias, residual = make_case(rng, n, R, H, scale=0.01)          # small values: the fp64 sum is exact
    whole, kept = oracle.mp_epilogue(partials, bias, residual, 0, p, seed)
    cuts = [0, 8, 1000, 1008, 4096, n]
    parts = [oracle.mp_epilogue([x[a:b].copy() for x in partials], bias, residual[a:b].copy(), a, p, seed)[0]
             for a, b in zip(cuts[:-1], cuts[1:])]
    assert np.array_equal(whole, np.concatenate(parts))
    perm = [partials[i] for i in rng.permutation(R)]
    assert np.array_equal(oracle.mp_epilogue(perm, bias, residual, 0, p, seed)[0], whole)
    # p close to 1 keeps almost nothing, and what it keeps is scaled by 1/(1-p)
    out, k = oracle.mp_epilogue(partials, bias, residual, 0, 0.999, seed)
    assert k.mean() < 0.01
