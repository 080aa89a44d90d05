"""GPU-vs-oracle comparison used by the gpu tests: same seeded bits on both sides, element by element.

The GPU side runs through the C ABI (paper_2105_05720_amd.binding); the oracle side runs oracle/ on the host.
Each side carries its own state from step to step; nothing the GPU computed is ever fed to the oracle.
"""
from __future__ import annotations

import os
from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from util import REL_TOL, half_ulp_distance, state_error

THREADS = min(16, len(os.sched_getaffinity(0)))


def to_np_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().astype(np.float32, copy=True)


def to_np_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16).copy()


def grad_to_np(shard: Shard, t: torch.Tensor) -> np.ndarray:
    """A gradient slice as the oracle takes it: uint16 bit patterns for fp16 slices, float32 for fp32 slices."""
    return to_np_bits(t) if shard.grad_dtype == torch.float16 else to_np_f32(t)


def hyper_pair(**kw):
    """The same step scalars for both sides (two separate dataclasses; neither package imports the other)."""
    return cc.Hyper(**kw), oracle.Hyper(**kw)


class OracleState:
    """Host-side fp32 state of the chosen tensors, advanced only by the oracle."""

    def __init__(self, shard: Shard, which: Sequence[int]):
        self.which = list(which)
        self.w = {k: to_np_f32(shard.w_of(k)) for k in self.which}
        self.m = {k: to_np_f32(shard.m_of(k)) for k in self.which}
        self.v = {k: to_np_f32(shard.v_of(k)) for k in self.which}
        self.w16 = {k: to_np_bits(shard.w16_of(k)) for k in self.which}

    def tensors(self, shard: Shard) -> List[oracle.OracleTensor]:
        return [oracle.OracleTensor(w=self.w[k], m=self.m[k], v=self.v[k],
                                    grads=[grad_to_np(shard, shard.grad_of(r, k)) for r in range(shard.R)],
                                    weight_decay=shard.wds[k]) for k in self.which]

    def adopt(self, ots: List[oracle.OracleTensor]):
        for k, t in zip(self.which, ots):
            self.w[k], self.m[k], self.v[k], self.w16[k] = t.w_out, t.m_out, t.v_out, t.w16_out


def compare_committed(shard: Shard, ost: OracleState, label: str, check_w16: bool = True):
    """Committed GPU state against the oracle's, tensor by tensor, to the parity bar."""
    worst = {"w": 0.0, "m": 0.0, "v": 0.0}
    worst_rel = {"w": 0.0, "m": 0.0, "v": 0.0}
    for k in ost.which:
        for name, got, want in (("w", shard.w_of(k), ost.w[k]), ("m", shard.m_of(k), ost.m[k]),
                                ("v", shard.v_of(k), ost.v[k])):
            ratio, rel, cnt = state_error(to_np_f32(got), want)
            worst[name] = max(worst[name], ratio)
            worst_rel[name] = max(worst_rel[name], rel)
            assert ratio <= 1.0, "%s: tensor %d %s off by %.3g x the %.0e bound (max rel %.3g, %d elements above)" % (
                label, k, name, ratio, REL_TOL, rel, cnt)
        if check_w16:
            d = half_ulp_distance(to_np_bits(shard.w16_of(k)), ost.w16[k])
            assert d.size == 0 or d.max() <= 1, "%s: tensor %d fp16 weights differ by %d ulp" % (label, k, d.max())
    return worst, worst_rel


def all_inputs_finite(shard: Shard) -> bool:
    """Independent scan of every gradient arena with torch (a library routine, not the library under test)."""
    return all(bool(torch.isfinite(g).all().item()) for g in shard.grads)


def run_steps(shard: Shard, ost: OracleState, gpu_fn: Callable, oracle_fn: Callable, hps, label: str,
              fill_grads: Callable[[int], None], expect_flags: Optional[Sequence[int]] = None,
              check_untouched: bool = True, same_start: bool = False):
    """hps: one (gpu hyper, oracle hyper) pair per call.  fill_grads(i) writes the i-th call's gradients.
    same_start: before every call the oracle takes over the GPU's committed fp32 state, so that each step is compared
    from identical inputs; otherwise both sides follow their own trajectory and the differences of earlier steps stay in.

    When the oracle holds only part of the tensor list, every non-finite input must sit in a tensor it holds
    (the tests arrange that and confirm it with all_inputs_finite on the other calls).
    """
    report = []
    for i, (ghp, ohp) in enumerate(hps):
        fill_grads(i)
        torch.cuda.synchronize()
        if same_start:
            for k in ost.which:
                ost.w[k], ost.m[k], ost.v[k] = (to_np_f32(x).copy() for x in (shard.w_of(k), shard.m_of(k), shard.v_of(k)))
        ots = ost.tensors(shard)
        oflag = oracle_fn(ots, ohp, threads=THREADS)
        before = shard.cur
        snap = None
        if check_untouched and not shard.in_place:
            snap = [(shard.w_of(k).clone(), shard.m_of(k).clone(), shard.v_of(k).clone(), shard.w16_of(k).clone())
                    for k in ost.which]
        gflag = shard.step(gpu_fn, ghp)
        torch.cuda.synchronize()
        assert gflag == oflag, "%s call %d: overflow flag %d, oracle %d" % (label, i, gflag, oflag)
        if expect_flags is not None:
            assert gflag == expect_flags[i], "%s call %d: flag %d, expected %d" % (label, i, gflag, expect_flags[i])
        if gflag and ghp.skip_mode == 0:
            assert shard.cur == before          # the written copy was not adopted
            if snap is not None:                # and the committed copy is bit-for-bit what it was
                for k, (w0, m0, v0, h0) in zip(ost.which, snap):
                    assert torch.equal(w0, shard.w_of(k)) and torch.equal(m0, shard.m_of(k))
                    assert torch.equal(v0, shard.v_of(k)) and torch.equal(h0.view(torch.int16), shard.w16_of(k).view(torch.int16))
        ost.adopt(ots)                          # a skipped oracle step returns its inputs
        report.append(compare_committed(shard, ost, "%s call %d" % (label, i)))
    return report


def seeded_state(shard: Shard, seed: int, with_history: bool = True, w_std: float = 0.02):
    """Random committed state: w ~ N(0, w_std), and (optionally) a plausible m, v history; w16 = fp16(w)."""
    g = torch.Generator(device=shard.device)
    g.manual_seed(seed)
    c = shard.cur
    shard.w[c].normal_(0.0, w_std, generator=g)
    if with_history:
        shard.m[c].normal_(0.0, 3e-3, generator=g)
        shard.v[c].normal_(0.0, 1e-3, generator=g)
        shard.v[c].square_()
    else:
        shard.m[c].zero_()
        shard.v[c].zero_()
    shard.w16[c].copy_(shard.w[c])


def seeded_grads(shard: Shard, seed: int, std: float):
    """All R gradient arenas: fp16(N(0, std)), one generator seed per rank."""
    for r, arena in enumerate(shard.grads):
        g = torch.Generator(device=shard.device)
        g.manual_seed(seed * 1000 + r)
        tmp = torch.empty(arena.numel(), dtype=torch.float32, device=shard.device)
        tmp.normal_(0.0, std, generator=g)
        arena.copy_(tmp)


# ---- full-size comparison: the oracle over EVERY element, streamed in batches; the comparison itself runs on the device ----

def device_state_ratio(got: torch.Tensor, want_np: np.ndarray):
    """state_error() of util.py evaluated with torch on the device (a library routine as test plumbing, float64):
    (worst |x-y| / (REL_TOL max(|y|, rms(y))), worst pure relative error)."""
    if got.numel() == 0:
        return 0.0, 0.0
    y = torch.from_numpy(want_np).to(got.device).double()
    x = got.double()
    fx, fy = torch.isfinite(x), torch.isfinite(y)
    if not torch.equal(fx, fy):
        return float("inf"), float("inf")
    x, y = x[fy], y[fy]
    if x.numel() == 0:
        return 0.0, 0.0
    rms = torch.sqrt(torch.mean(y * y))
    diff = (x - y).abs()
    floor = torch.maximum(y.abs(), rms)
    ratio = diff / (REL_TOL * torch.where(floor > 0, floor, torch.ones_like(floor)))
    ratio = torch.where((floor == 0) & (diff == 0), torch.zeros_like(ratio), ratio)
    rel = torch.where(y != 0, diff / y.abs(), torch.where(diff == 0, torch.zeros_like(diff), torch.full_like(diff, float("inf"))))
    return float(ratio.max().item()), float(rel.max().item())


def device_half_ulp_max(got_half: torch.Tensor, want_bits_np: np.ndarray) -> int:
    """Largest distance on the ordered fp16 line between two sets of bit patterns (two non-finite values are equal)."""
    if got_half.numel() == 0:
        return 0
    a = got_half.view(torch.int16).to(torch.int64) & 0xFFFF
    b = torch.from_numpy(want_bits_np.view(np.int16)).to(got_half.device).to(torch.int64) & 0xFFFF

    def key(x):
        mag = x & 0x7FFF
        return torch.where((x & 0x8000) != 0, -mag, mag)
    d = (key(a) - key(b)).abs()
    both = ((a & 0x7C00) == 0x7C00) & ((b & 0x7C00) == 0x7C00)
    return int(torch.where(both, torch.zeros_like(d), d).max().item())


class FullOracle:
    """The oracle's own fp32 state of EVERY tensor of a shard on the host, advanced only by the oracle.  A step pulls the
    gradients from the device batch by batch (they are the seeded inputs both sides read), runs the oracle on each batch
    and keeps the new state aside until the flag of the whole step is known (whole-step skip spans all tensors)."""

    def __init__(self, shard: Shard, batch_elems: int = 160_000_000, piece_elems: int = 8_000_000):
        self.T = len(shard.numels)
        self.w = [to_np_f32(shard.w_of(k)) for k in range(self.T)]
        self.m = [to_np_f32(shard.m_of(k)) for k in range(self.T)]
        self.v = [to_np_f32(shard.v_of(k)) for k in range(self.T)]
        self.w16 = [to_np_bits(shard.w16_of(k)) for k in range(self.T)]
        self.norms = [None] * self.T
        self.piece_elems = piece_elems
        self.batches, cur, size = [], [], 0
        for k, n in enumerate(shard.numels):
            if cur and size + n > batch_elems:
                self.batches.append(cur)
                cur, size = [], 0
            cur.append(k)
            size += n
        if cur:
            self.batches.append(cur)
        self.elements = sum(shard.numels)

    def step(self, shard: Shard, ohp, optimizer: str) -> int:
        """One oracle step over all tensors.  Returns the flag; on a skipped step the state stays as it was."""
        new = {}
        flag = 0
        for batch in self.batches:
            grads = {k: [grad_to_np(shard, shard.grad_of(r, k)) for r in range(shard.R)] for k in batch}
            ots, owner = [], []
            for k in batch:
                n = self.w[k].size
                # Adam is independent per element: a huge tensor is handed over in pieces so that all host threads work
                # on it; a LAMB tensor is one trust-ratio unit and stays whole
                step_n = self.piece_elems if (optimizer == "adam" and n > self.piece_elems) else max(n, 1)
                for a in range(0, max(n, 1), step_n):
                    b = min(n, a + step_n)
                    ots.append(oracle.OracleTensor(w=self.w[k][a:b], m=self.m[k][a:b], v=self.v[k][a:b],
                                                   grads=[g[a:b] for g in grads[k]], weight_decay=shard.wds[k]))
                    owner.append(k)
            f = (oracle.adam_step if optimizer == "adam" else oracle.lamb_step)(ots, ohp, threads=THREADS)
            flag |= f
            for k in batch:
                mine = [t for t, o in zip(ots, owner) if o == k]
                cat = (lambda xs: xs[0] if len(xs) == 1 else np.concatenate(xs))
                new[k] = (cat([t.w_out for t in mine]), cat([t.m_out for t in mine]), cat([t.v_out for t in mine]),
                          cat([t.w16_out for t in mine]), mine[0].norms if optimizer == "lamb" else None)
        if flag and ohp.skip_mode == 0:
            return flag                         # every tensor keeps its state, also those of batches without an inf/NaN
        for k, (w, m, v, h, norms) in new.items():
            self.w[k], self.m[k], self.v[k], self.w16[k], self.norms[k] = w, m, v, h, norms
        return flag

    def compare(self, shard: Shard, label: str):
        """Every element of the committed device state against the oracle's, to the parity bar.  Returns the worst
        ratio to the bound over all tensors."""
        worst = 0.0
        for k in range(self.T):
            for name, got, want in (("w", shard.w_of(k), self.w[k]), ("m", shard.m_of(k), self.m[k]), ("v", shard.v_of(k), self.v[k])):
                ratio, rel = device_state_ratio(got, want)
                worst = max(worst, ratio)
                assert ratio <= 1.0, "%s: tensor %d %s off by %.3g x the %.0e bound (max rel %.3g)" % (label, k, name, ratio, REL_TOL, rel)
            d = device_half_ulp_max(shard.w16_of(k), self.w16[k])
            assert d <= 1, "%s: tensor %d fp16 weights differ by %d ulp" % (label, k, d)
        return worst
