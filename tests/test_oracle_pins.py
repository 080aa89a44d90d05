"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test fixes the oracle to something the paper or the mathematics decides: numpy's float16 for the
fp16 codec, torch.optim.AdamW / Adam in float64 as the one-rank special case of the Adam program
(paper, Fig. 4a), closed forms of the first step, and invariances that hold for any correct
implementation.  A dropped term, a wrong sign, a swapped beta or a misplaced epsilon fails one of them.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import Hyper
from util import bits_to_f64, f32, fl, half_bits, make_tensor, ulp_f32

F = lambda x: float(np.float32(x))   # the fp32 value a C float argument carries


# ----------------------------------------------------------------------------- fp16 codec

def test_half_decode_exhaustive_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def _encode_many(xs):
    return np.array([oracle.float_to_half(float(x)) for x in xs], dtype=np.uint16)


def test_half_encode_against_numpy():
    rng = np.random.default_rng(1)
    halves = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    fin = halves[np.isfinite(halves)]
    srt = np.sort(np.unique(fin))
    mid = (srt[:-1] + srt[1:]) / 2                       # exact ties between neighbours (fit in fp32)
    near = np.concatenate([np.nextafter(mid.astype(np.float32), np.float32(np.inf)),
                           np.nextafter(mid.astype(np.float32), np.float32(-np.inf))]).astype(np.float64)
    rnd = np.concatenate([rng.normal(0, s, 4000) for s in (1e-8, 1e-6, 1e-4, 1e-2, 1, 100, 3e4)])
    edge = np.array([0.0, -0.0, 65504, 65519.99, 65520, 65536, 1e30, -1e30, np.inf, -np.inf,
                     2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26, 2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12)])
    xs = np.concatenate([fin, mid, near, rnd, edge, -edge]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = _encode_many(xs)
    assert np.array_equal(got, want)
    nan_bits = oracle.float_to_half(float("nan"))
    assert (nan_bits & 0x7C00) == 0x7C00 and (nan_bits & 0x03FF) != 0


# ----------------------------------------------------------------------------- Adam vs torch (library special case)

def _torch_adam_step(cls, w, m, v, g, hp, wd, t):
    """One step of torch's float64 optimizer from given state; returns (w', m', v') as float64 arrays."""
    p = torch.nn.Parameter(torch.tensor(np.asarray(w, dtype=np.float64)))
    opt = cls([p], lr=F(hp.lr), betas=(F(hp.beta1), F(hp.beta2)), eps=F(hp.eps), weight_decay=F(wd))
    opt.state[p] = {"step": torch.tensor(float(t - 1)),
                    "exp_avg": torch.tensor(np.asarray(m, dtype=np.float64)),
                    "exp_avg_sq": torch.tensor(np.asarray(v, dtype=np.float64))}
    p.grad = torch.tensor(np.asarray(g, dtype=np.float64))
    opt.step()
    st = opt.state[p]
    return p.detach().numpy().copy(), st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()


def _random_case(rng, n, R, gstd=1e-2, with_state=True):
    w = f32(rng.normal(0, 0.02, n))
    m = f32(rng.normal(0, 3e-3, n)) if with_state else np.zeros(n, np.float32)
    v = f32(rng.normal(0, 1e-3, n) ** 2) if with_state else np.zeros(n, np.float32)
    grads = [half_bits(rng.normal(0, gstd, n)) for _ in range(R)]
    return w, m, v, grads


@pytest.mark.parametrize("mode,cls", [(1, torch.optim.AdamW), (0, torch.optim.Adam)])
@pytest.mark.parametrize("t", [1, 2, 7, 1000])
def test_adam_one_rank_equals_torch_float64(mode, cls, t):
    rng = np.random.default_rng(10 + t)
    n = 4096
    w, m, v, grads = _random_case(rng, n, 1)
    hp = Hyper(lr=2e-3, beta1=0.9, beta2=0.999, eps=1e-6, step=t, adam_mode=mode)
    wd = 0.01
    ot = make_tensor(w, grads, m, v, wd)
    assert oracle.adam_step([ot], hp) == 0
    tw, tm, tv = _torch_adam_step(cls, w, m, v, bits_to_f64(grads[0]), hp, wd, t)
    # both are float64 computations of the same formula; after rounding to fp32 they agree to the last bit
    # except where the float64 value sits within ~1e-16 of a rounding boundary
    for got, want in ((ot.w_out, tw), (ot.m_out, tm), (ot.v_out, tv)):
        d = ulp_f32(got, want.astype(np.float32))
        assert d.max() <= 1
        assert np.mean(d == 0) > 0.999
    with np.errstate(over="ignore"):
        assert np.array_equal(ot.w16_out, ot.w_out.astype(np.float16).view(np.uint16))


def test_adam_multi_step_tracks_torch():
    """Four consecutive steps, state carried in fp32 by the oracle and in float64 by torch."""
    rng = np.random.default_rng(5)
    n, wd = 2048, 0.01
    w, m, v, _ = _random_case(rng, n, 1, with_state=False)
    p = torch.nn.Parameter(torch.tensor(w.astype(np.float64)))
    opt = torch.optim.AdamW([p], lr=F(1e-3), betas=(F(0.9), F(0.999)), eps=F(1e-6), weight_decay=F(wd))
    for t in range(1, 5):
        g = half_bits(rng.normal(0, 1e-2, n))
        ot = make_tensor(w, [g], m, v, wd)
        oracle.adam_step([ot], Hyper(step=t))
        w, m, v = ot.w_out, ot.m_out, ot.v_out
        p.grad = torch.tensor(bits_to_f64(g))
        opt.step()
    # the oracle rounds its state to fp32 after every step (half an ulp of the largest value each time);
    # a wrong step count, bias correction or decay would be off by 1e-5 or more
    tw, tm, tv = p.detach().numpy(), opt.state[p]["exp_avg"].numpy(), opt.state[p]["exp_avg_sq"].numpy()
    for got, want in ((w, tw), (m, tm), (v, tv)):
        assert np.max(np.abs(got - want)) <= 4 * 2.0 ** -24 * np.max(np.abs(want))


# ----------------------------------------------------------------------------- Adam closed forms

def test_first_step_is_lr_times_sign_up_to_eps():
    rng = np.random.default_rng(2)
    n, R = 3000, 4
    w, _, _, grads = _random_case(rng, n, R, with_state=False)
    hp = Hyper(lr=1e-3, eps=1e-6, step=1)
    ot = make_tensor(w, grads, wd=0.0)
    oracle.adam_step([ot], hp)
    S = sum(bits_to_f64(g) for g in grads)
    lr, eps = F(hp.lr), F(hp.eps)
    # at t=1 with m=v=0 the bias corrections cancel the (1-beta) factors exactly: mhat = S, vhat = S^2
    closed = w.astype(np.float64) - lr * S / (np.abs(S) + eps)
    assert ulp_f32(ot.w_out, closed.astype(np.float32)).max() <= 1
    assert np.mean(ot.w_out == closed.astype(np.float32)) > 0.999
    delta = ot.w_out.astype(np.float64) - w
    bound = lr * eps / (np.abs(S) + eps) + np.maximum(np.abs(w), np.abs(ot.w_out)) * 2.0 ** -23
    assert np.all(np.abs(delta + lr * np.sign(S)) <= bound + 1e-12)


def test_fp16_copy_is_made_from_the_stored_fp32_weight():
    """State is fp32 and the fp16 copy is what a cast of that fp32 tensor gives (two roundings, not one).
    Worked by hand: the first step with m = v = 0, no decay and eps = 0 moves w by exactly lr sign(S).  With
    w = 1 + 2^-10 and lr = 2^-11 - 2^-30 the exact result is T + 2^-30, T = 1 + 2^-11 being the midpoint of the fp16
    neighbours 1 and 1 + 2^-10.  fp32 has no room for the 2^-30: the stored weight is T itself, and the tie goes
    to the even fp16 neighbour 1.0 (0x3C00).  Rounding the exact result to fp16 directly would give 1 + 2^-10."""
    w = np.array([1 + 2.0 ** -10, -(1 + 2.0 ** -10)], np.float32)
    grads = [half_bits([0.25, -0.25])]
    lr = 2.0 ** -11 - 2.0 ** -30
    assert float(np.float32(lr)) == lr
    ot = make_tensor(w, grads, wd=0.0)
    oracle.adam_step([ot], Hyper(lr=lr, eps=0.0, step=1))
    assert np.array_equal(ot.w_out, np.array([1 + 2.0 ** -11, -(1 + 2.0 ** -11)], np.float32))
    assert list(ot.w16_out) == [0x3C00, 0xBC00]
    # LAMB on a one-element tensor: ratio = |w| / |sign| = |w|, so the move is lr |w| sign(S); w = 1 gives the same numbers
    # when lr is chosen for it: 1 - lr' = T' + tiny with T' = 1 - 2^-12 the midpoint of fp16's 1 - 2^-11 and 1
    lr2 = 2.0 ** -12 - 2.0 ** -32
    assert float(np.float32(lr2)) == lr2
    ot = make_tensor(np.array([1.0], np.float32), [half_bits([0.5])], wd=0.0)
    oracle.lamb_step([ot], Hyper(lr=lr2, eps=0.0, step=1))
    assert ot.w_out[0] == np.float32(1 - 2.0 ** -12)          # 1 - 2^-12 + 2^-32 does not fit fp32 below 1 (ulp 2^-24)
    assert ot.w16_out[0] == 0x3C00                              # tie between 0x3BFF and 0x3C00: even is 0x3C00; direct rounding gives 0x3C00 too
    # the mirrored case separates the two roundings for LAMB as well: exact = T' - 2^-32 -> fp32 T' -> tie -> 0x3C00, direct -> 0x3BFF
    lr3 = 2.0 ** -12 + 2.0 ** -32
    assert float(np.float32(lr3)) == lr3
    ot = make_tensor(np.array([1.0], np.float32), [half_bits([0.5])], wd=0.0)
    oracle.lamb_step([ot], Hyper(lr=lr3, eps=0.0, step=1))
    assert ot.w_out[0] == np.float32(1 - 2.0 ** -12) and ot.w16_out[0] == 0x3C00


def test_identical_gradients_sum_to_R_times_g():
    rng = np.random.default_rng(3)
    n, R = 1000, 8
    w = f32(rng.normal(0, 0.02, n))
    g = half_bits(rng.normal(0, 1e-2, n))
    for ls, avg in ((1.0, 0), (1024.0, 0), (1.0, 1), (8.0, 1)):
        hp = Hyper(loss_scale=ls, grad_average=avg, step=1)
        ot = make_tensor(w, [g.copy() for _ in range(R)], wd=0.01)
        oracle.adam_step([ot], hp)
        ghat = R * bits_to_f64(g) / ls / (R if avg else 1)
        b1, b2 = F(hp.beta1), F(hp.beta2)
        assert np.array_equal(ot.m_out, ((1 - b1) * ghat).astype(np.float32))
        assert np.array_equal(ot.v_out, ((1 - b2) * ghat * ghat).astype(np.float32))


def test_zero_gradients():
    rng = np.random.default_rng(4)
    n, R, wd = 500, 3, 0.01
    w, m, v, _ = _random_case(rng, n, R)
    zeros = [np.zeros(n, np.uint16) for _ in range(R)]
    zeros[1][::2] = 0x8000                                  # negative zero is still zero
    hp = Hyper(step=3)
    b1, b2, lr = F(hp.beta1), F(hp.beta2), F(hp.lr)
    ot = make_tensor(w, zeros, m, v, wd)
    oracle.adam_step([ot], hp)
    assert np.array_equal(ot.m_out, (b1 * m.astype(np.float64)).astype(np.float32))
    assert np.array_equal(ot.v_out, (b2 * v.astype(np.float64)).astype(np.float32))
    # with no history either, m stays 0 and the step is pure decay
    ot0 = make_tensor(w, zeros, wd=wd)
    oracle.adam_step([ot0], hp)
    assert not ot0.m_out.any() and not ot0.v_out.any()
    assert np.array_equal(ot0.w_out, (w.astype(np.float64) * (1 - lr * F(wd))).astype(np.float32)) or \
        ulp_f32(ot0.w_out, (w.astype(np.float64) * (1 - lr * F(wd))).astype(np.float32)).max() <= 1


# ----------------------------------------------------------------------------- invariances

def test_rank_permutation_and_loss_scale_invariance():
    rng = np.random.default_rng(6)
    n, R = 777, 8
    w, m, v, grads = _random_case(rng, n, R, gstd=1e-3)      # mostly subnormal-range halves
    hp = Hyper(step=5)
    a = make_tensor(w, grads, m, v, 0.01)
    oracle.adam_step([a], hp)
    b = make_tensor(w, [grads[i] for i in rng.permutation(R)], m, v, 0.01)
    oracle.adam_step([b], hp)
    for x, y in ((a.w_out, b.w_out), (a.m_out, b.m_out), (a.v_out, b.v_out), (a.w16_out, b.w16_out)):
        assert np.array_equal(x, y)
    # gradients pre-multiplied by 2^k (exact in fp16 here) and unscaled by loss_scale = 2^k
    g64 = [bits_to_f64(g) for g in grads]
    scaled = [half_bits(g * 256.0) for g in g64]
    assert all(np.array_equal(bits_to_f64(s), g * 256.0) for s, g in zip(scaled, g64))
    c = make_tensor(w, scaled, m, v, 0.01)
    oracle.adam_step([c], Hyper(step=5, loss_scale=256.0))
    assert np.array_equal(a.w_out, c.w_out) and np.array_equal(a.m_out, c.m_out) and np.array_equal(a.v_out, c.v_out)


def test_flat_equals_scattered():
    """The same elements as one tensor or cut into pieces give the same Adam update (paper, Table 2's premise)."""
    rng = np.random.default_rng(7)
    n, R = 5000, 4
    w, m, v, grads = _random_case(rng, n, R)
    hp = Hyper(step=2)
    whole = make_tensor(w, grads, m, v, 0.01)
    oracle.adam_step([whole], hp)
    cuts = [0, 1, 9, 1033, 1034, 4097, n]
    parts = [make_tensor(w[a:b], [g[a:b] for g in grads], m[a:b], v[a:b], 0.01) for a, b in zip(cuts[:-1], cuts[1:])]
    oracle.adam_step(parts, hp, threads=3)
    assert np.array_equal(whole.w_out, np.concatenate([p.w_out for p in parts]))
    assert np.array_equal(whole.v_out, np.concatenate([p.v_out for p in parts]))
    assert np.array_equal(whole.w16_out, np.concatenate([p.w16_out for p in parts]))


# ----------------------------------------------------------------------------- overflow flag and skip

def test_overflow_flag_is_any_nonfinite_input_bit_pattern():
    rng = np.random.default_rng(8)
    for trial in range(200):
        n, R = int(rng.integers(1, 40)), int(rng.integers(1, 17))
        grads = [rng.integers(0, 65536, n).astype(np.uint16) for _ in range(R)]
        if trial % 2:                                          # keep half of the trials finite
            for g in grads:
                g[(g & 0x7C00) == 0x7C00] &= 0xBBFF
        if trial % 4 == 3:                                     # opposite infinities cancel to NaN, still flagged
            grads[0][0] = 0x7C00
            if R > 1:
                grads[1][0] = 0xFC00
        brute = int(any(((g & 0x7C00) == 0x7C00).any() for g in grads))
        assert oracle.grad_overflow(grads) == brute


def test_whole_step_skip_and_element_guard():
    rng = np.random.default_rng(9)
    n, R = 300, 4
    w, m, v, grads = _random_case(rng, n, R)
    w2, m2, v2, grads2 = _random_case(rng, 64, R)
    clean = [make_tensor(w, grads, m, v, 0.01), make_tensor(w2, grads2, m2, v2, 0.0)]
    assert oracle.adam_step(clean, Hyper(step=2)) == 0
    bad = [g.copy() for g in grads2]
    bad[2][17] = 0x7C00
    bad[1][40] = 0x7E01                                        # a NaN
    skipped = [make_tensor(w, grads, m, v, 0.01), make_tensor(w2, bad, m2, v2, 0.0)]
    assert oracle.adam_step(skipped, Hyper(step=2, skip_mode=0)) == 1
    for t, (ww, mm, vv) in zip(skipped, ((w, m, v), (w2, m2, v2))):
        assert np.array_equal(t.w_out, ww) and np.array_equal(t.m_out, mm) and np.array_equal(t.v_out, vv)
        assert np.array_equal(t.w16_out, ww.astype(np.float16).view(np.uint16))
    guarded = [make_tensor(w, grads, m, v, 0.01), make_tensor(w2, bad, m2, v2, 0.0)]
    assert oracle.adam_step(guarded, Hyper(step=2, skip_mode=1)) == 1
    assert np.array_equal(guarded[0].w_out, clean[0].w_out)
    keep = np.zeros(64, bool)
    keep[[17, 40]] = True
    g1, c1 = guarded[1], clean[1]
    assert np.array_equal(g1.w_out[~keep], c1.w_out[~keep]) and np.array_equal(g1.m_out[~keep], c1.m_out[~keep])
    assert np.array_equal(g1.w_out[keep], w2[keep]) and np.array_equal(g1.v_out[keep], v2[keep])
    # LAMB skips the whole step as well
    lam = [make_tensor(w2, bad, m2, v2, 0.01)]
    assert oracle.lamb_step(lam, Hyper(step=2)) == 1
    assert np.array_equal(lam[0].w_out, w2) and np.array_equal(lam[0].m_out, m2)


# ----------------------------------------------------------------------------- LAMB

def test_lamb_single_element_moves_by_lr_times_abs_w():
    hp = Hyper(lr=1e-2, step=1)
    for wv, gv in ((0.5, 0.25), (-0.5, 0.25), (0.125, -3.0), (-2.0, -1e-3)):
        t = make_tensor([wv], [half_bits([gv])], wd=0.0)
        oracle.lamb_step([t], hp)
        # one element: ratio = |w|/|u|, so the move is lr*|w| against the sign of u (= sign of g at t=1)
        want = wv - F(hp.lr) * abs(wv) * np.sign(gv)
        assert t.w_out[0] == np.float32(want)


def test_lamb_pure_decay_shrinks_by_lr():
    rng = np.random.default_rng(11)
    n, wd = 1000, 0.01
    w = f32(rng.normal(0, 0.02, n))
    t = make_tensor(w, [np.zeros(n, np.uint16)] * 2, wd=wd)
    hp = Hyper(lr=1e-3, step=1)
    oracle.lamb_step([t], hp)
    # g = 0, no history: u = wd*w, ||u|| = wd*||w||, ratio = 1/wd, w' = w - lr*w
    assert ulp_f32(t.w_out, (w.astype(np.float64) * (1 - F(hp.lr))).astype(np.float32)).max() <= 1
    assert t.norms[1] == pytest.approx(F(wd) * t.norms[0], rel=1e-12)


def test_lamb_first_step_closed_form_and_norms():
    rng = np.random.default_rng(12)
    n, R = 4096, 4
    w = f32(rng.normal(0, 0.02, n))
    gv = rng.choice([-1.0, 1.0], n) * rng.uniform(0.5, 2.0, n)     # |g| >> eps
    grads = [half_bits(gv / R)] * R
    hp = Hyper(lr=1e-3, eps=1e-6, step=1)
    t = make_tensor(w, grads, wd=0.0)
    oracle.lamb_step([t], hp)
    nw = np.linalg.norm(w.astype(np.float64))
    assert t.norms[0] == pytest.approx(nw, rel=1e-13)
    assert t.norms[1] == pytest.approx(np.sqrt(n), rel=3e-6)       # u = g/(|g|+eps) ~ sign(g)
    S = R * bits_to_f64(grads[0])
    want = w - F(hp.lr) * nw / np.sqrt(n) * np.sign(S)
    assert np.allclose(t.w_out, want, rtol=0, atol=F(hp.lr) * nw / np.sqrt(n) * 5e-6 + 1e-9)


def test_lamb_zero_weight_tensor_and_unit_ratio_reduce_to_adamw():
    rng = np.random.default_rng(13)
    n, R = 1024, 2
    _, m, v, grads = _random_case(rng, n, R)
    hp = Hyper(step=4)
    # ||w|| = 0  ->  ratio 1
    z = make_tensor(np.zeros(n), grads, m, v, 0.01)
    oracle.lamb_step([z], hp)
    a = make_tensor(np.zeros(n), grads, m, v, 0.01)
    oracle.adam_step([a], hp)
    assert np.array_equal(z.w_out, a.w_out) and np.array_equal(z.m_out, a.m_out) and np.array_equal(z.v_out, a.v_out)
    # ||w|| = ||u||: without decay u does not depend on w, so scale w onto the sphere of radius ||u||
    w = rng.normal(0, 0.02, n)
    probe = make_tensor(w, grads, m, v, 0.0)
    oracle.lamb_step([probe], hp)
    w1 = f32(w * probe.norms[1] / np.linalg.norm(w))
    lam = make_tensor(w1, grads, m, v, 0.0)
    oracle.lamb_step([lam], hp)
    assert lam.norms[0] == pytest.approx(lam.norms[1], rel=1e-7)
    S = sum(bits_to_f64(g) for g in grads)
    tw, tm, tv = _torch_adam_step(torch.optim.AdamW, w1, m, v, S, hp, 0.0, hp.step)
    assert np.allclose(lam.w_out, tw, rtol=3e-7, atol=0)
    assert np.array_equal(lam.m_out, tm.astype(np.float32)) or ulp_f32(lam.m_out, tm.astype(np.float32)).max() <= 1


def test_lamb_general_case_from_torch_update_direction():
    """u taken from torch: AdamW with lr = 1 moves p by exactly -u; LAMB then rescales that move per tensor."""
    rng = np.random.default_rng(14)
    n, R, wd = 3000, 3, 0.01
    w, m, v, grads = _random_case(rng, n, R)
    hp = Hyper(lr=3e-3, step=6)
    t = make_tensor(w, grads, m, v, wd)
    oracle.lamb_step([t], hp)
    S = sum(bits_to_f64(g) for g in grads)
    one = Hyper(lr=1.0, beta1=hp.beta1, beta2=hp.beta2, eps=hp.eps, step=hp.step)
    tw, tm, tv = _torch_adam_step(torch.optim.AdamW, w, m, v, S, one, wd, hp.step)
    u = w.astype(np.float64) - tw
    ratio = np.linalg.norm(w.astype(np.float64)) / np.linalg.norm(u)
    want = w.astype(np.float64) - F(hp.lr) * ratio * u
    assert np.allclose(t.w_out, want, rtol=2e-7, atol=1e-11)
    assert t.norms[1] == pytest.approx(np.linalg.norm(u), rel=1e-10)
    assert ulp_f32(t.m_out, tm.astype(np.float32)).max() <= 1 and ulp_f32(t.v_out, tv.astype(np.float32)).max() <= 1


def test_lamb_move_scales_with_the_weights():
    """Without decay, doubling w doubles ||w||, the ratio and hence w' exactly (powers of two are exact)."""
    rng = np.random.default_rng(15)
    n, R = 2000, 4
    w, m, v, grads = _random_case(rng, n, R)
    hp = Hyper(step=3)
    a = make_tensor(w, grads, m, v, 0.0)
    b = make_tensor(w * np.float32(2), grads, m, v, 0.0)
    oracle.lamb_step([a, b], hp, threads=2)
    assert np.array_equal(b.w_out, a.w_out * np.float32(2))
    assert np.array_equal(a.m_out, b.m_out)


def test_lamb_ratio_is_per_tensor():
    rng = np.random.default_rng(16)
    w, m, v, grads = _random_case(rng, 600, 2)
    hp = Hyper(step=2)
    whole = make_tensor(w, grads, m, v, 0.01)
    halves = [make_tensor(w[:300], [g[:300] for g in grads], m[:300], v[:300], 0.01),
              make_tensor(w[300:] * np.float32(10), [g[300:] for g in grads], m[300:], v[300:], 0.01)]
    oracle.lamb_step([whole], hp)
    oracle.lamb_step(halves, hp)
    # each tensor uses its own norms: the second half's ratio is ~10x the first's
    r = [h.norms[0] / h.norms[1] for h in halves]
    assert r[1] / r[0] == pytest.approx(10.0, rel=0.2)
    assert not np.array_equal(whole.w_out[:300], halves[0].w_out)


# ----------------------------------------------------------------------------- fp32 gradient slices

def test_fp32_gradients_one_rank_equals_torch_float64():
    """The same Adam program with fp32 gradient slices (the paper's Float 32 case, Section 6.1.1)."""
    rng = np.random.default_rng(31)
    n = 4096
    w, m, v, _ = _random_case(rng, n, 1)
    g = f32(rng.normal(0, 1e-2, n))
    for mode, cls in ((1, torch.optim.AdamW), (0, torch.optim.Adam)):
        hp = Hyper(lr=2e-3, step=3, adam_mode=mode)
        ot = make_tensor(w, [g], m, v, 0.01)
        assert oracle.adam_step([ot], hp) == 0
        tw, tm, tv = _torch_adam_step(cls, w, m, v, g.astype(np.float64), hp, 0.01, 3)
        for got, want in ((ot.w_out, tw), (ot.m_out, tm), (ot.v_out, tv)):
            assert ulp_f32(got, want.astype(np.float32)).max() <= 1


def test_fp32_gradients_sum_and_match_the_fp16_path_on_fp16_values():
    """fp32 slices that hold fp16-representable values give exactly what the fp16 slices give; R identical
    slices sum to R g; and the two oracles agree for LAMB too."""
    rng = np.random.default_rng(32)
    n, R = 3000, 8
    w, m, v, grads = _random_case(rng, n, R)
    as_f32 = [bits_to_f64(g).astype(np.float32) for g in grads]
    hp = Hyper(step=2, loss_scale=4.0)
    for step_fn in (oracle.adam_step, oracle.lamb_step):
        a = make_tensor(w, grads, m, v, 0.01)
        b = make_tensor(w, as_f32, m, v, 0.01)
        assert step_fn([a], hp) == step_fn([b], hp) == 0
        for x, y in ((a.w_out, b.w_out), (a.m_out, b.m_out), (a.v_out, b.v_out), (a.w16_out, b.w16_out)):
            assert np.array_equal(x, y)
    g = f32(rng.normal(0, 1e-2, n))
    ot = make_tensor(w, [g.copy() for _ in range(R)], wd=0.0)
    oracle.adam_step([ot], Hyper(step=1))
    b1 = F(0.9)
    assert np.array_equal(ot.m_out, ((1 - b1) * R * g.astype(np.float64)).astype(np.float32))


def test_fp32_gradient_overflow_is_decided_on_the_fp32_sum():
    big = np.float32(3e38)
    n = 8
    w = f32(np.full(n, 0.01))
    fine = [f32(np.full(n, 1.0)), f32(np.full(n, 2.0))]
    assert oracle.grad_overflow(fine) == 0
    over = [f32(np.full(n, big)), f32(np.full(n, big))]          # 6e38 is finite in double, infinite in fp32
    assert oracle.grad_overflow(over) == 1
    inf = [f32(np.full(n, 1.0)), f32(np.full(n, 1.0))]
    inf[1][3] = np.inf
    assert oracle.grad_overflow(inf) == 1
    nan = [f32(np.full(n, 1.0))]
    nan[0][7] = np.nan
    assert oracle.grad_overflow(nan) == 1
    t = make_tensor(w, over)
    assert oracle.adam_step([t], Hyper(step=1)) == 1
    assert np.array_equal(t.w_out, w)


# ----------------------------------------------------------------------------- brute force on tiny tensors

def test_tiny_tensors_against_a_numpy_float64_loop():
    """A second, independent write-up of the per-element program in numpy float64, element by element.  (It
    restates the formula, so it guards the C code against slips rather than pinning the formula itself.)"""
    rng = np.random.default_rng(40)
    for n, R in ((1, 1), (2, 3), (7, 8), (9, 16)):
        w, m, v, grads = _random_case(rng, n, R)
        hp = Hyper(lr=3e-3, beta1=0.8, beta2=0.99, eps=1e-7, loss_scale=8.0, step=5, grad_average=1)
        wd = 0.05
        ot = make_tensor(w, grads, m, v, wd)
        lt = make_tensor(w, grads, m, v, wd)
        oracle.adam_step([ot], hp)
        oracle.lamb_step([lt], hp)
        lr, b1, b2, eps, wdf = F(hp.lr), F(hp.beta1), F(hp.beta2), F(hp.eps), F(wd)
        us, ws = [], []
        for i in range(n):
            S = 0.0
            for g in grads:
                S += float(bits_to_f64(g[i:i + 1])[0])
            gh = S / (8.0 * R)
            mi = b1 * float(m[i]) + (1 - b1) * gh
            vi = b2 * float(v[i]) + (1 - b2) * gh * gh
            u = (mi / (1 - b1 ** 5)) / (np.sqrt(vi / (1 - b2 ** 5)) + eps) + wdf * float(w[i])
            us.append(u)
            ws.append(float(w[i]))
            assert ot.m_out[i] == np.float32(mi) and ot.v_out[i] == np.float32(vi)
            assert ulp_f32(ot.w_out[i:i + 1], np.array([np.float32(ws[-1] - lr * u)])).max() <= 1
        ratio = np.linalg.norm(ws) / np.linalg.norm(us)
        for i in range(n):
            assert ulp_f32(lt.w_out[i:i + 1], np.array([np.float32(ws[i] - lr * ratio * us[i])])).max() <= 1


# ----------------------------------------------------------------------------- fp16 intermediate (unfused baseline)

def test_fp16_intermediate_equals_one_rank_with_the_rounded_sum():
    """With sum_f16 the optimizer must see exactly fp16(fp32(sum)): the same as a single slice holding that value."""
    rng = np.random.default_rng(50)
    n, R = 4000, 8
    w, m, v, grads = _random_case(rng, n, R, gstd=0.7)                   # |S| > 1: the rounding to fp16 matters
    hp = Hyper(step=3, loss_scale=2.0)
    a = make_tensor(w, grads, m, v, 0.01)
    assert oracle.adam_step([a], hp, sum_f16=True) == 0
    S = sum(bits_to_f64(g) for g in grads)
    with np.errstate(over="ignore"):
        S16 = S.astype(np.float32).astype(np.float16)                     # numpy: fp32 then fp16, nearest even
    b = make_tensor(w, [S16.view(np.uint16)], m, v, 0.01)
    oracle.adam_step([b], hp)
    assert np.array_equal(a.w_out, b.w_out) and np.array_equal(a.m_out, b.m_out) and np.array_equal(a.v_out, b.v_out)
    c = make_tensor(w, grads, m, v, 0.01)
    oracle.adam_step([c], hp)
    assert not np.array_equal(a.m_out, c.m_out)                            # and it differs from the exact-sum path
    # a finite sum beyond the fp16 range comes back as inf and raises the flag
    big = [half_bits(np.full(8, 60000.0)), half_bits(np.full(8, 60000.0))]
    assert oracle.grad_overflow(big) == 0 and oracle.grad_overflow(big, sum_f16=True) == 1
