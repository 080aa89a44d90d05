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
              check_untouched: bool = True):
    """hps: one (gpu hyper, oracle hyper) pair per call.  fill_grads(i) writes the i-th call's gradients.

    When the oracle holds only part of the tensor list, every non-finite input must sit in a tensor it holds
    (the tests arrange that and confirm it with all_inputs_finite on the other calls).
    """
    report = []
    for i, (ghp, ohp) in enumerate(hps):
        fill_grads(i)
        torch.cuda.synchronize()
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
