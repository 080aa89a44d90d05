"""The five benchmark configurations at full size, in the launch configuration bench.py times (default chunk
size, out-of-place state), checked against the oracle on what it can compute in seconds:

  Adam (configs 1, 2, 4): the update is independent per element, so the oracle recomputes a strided sample of
  every tensor (every STRIDE-th element plus each tensor's last 9, which covers the scalar tail) and a few
  whole tensors; config 1 is small enough to be recomputed whole.
  LAMB (configs 3, 5): the trust ratio needs whole tensors, so the oracle recomputes a subset of whole tensors
  (tensors are independent of each other).
  Everything else is covered by properties that hold at any size: the flag, untouched inputs on a skipped step,
  and bit-equality of the fused result with the unfused pipeline over all elements.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd import workloads as W
from paper_2105_05720_amd.shard import Shard
from parity import (THREADS, OracleState, all_inputs_finite, compare_committed, grad_to_np, hyper_pair, run_steps, to_np_bits,
                    to_np_f32)
from util import half_ulp_distance, state_error

pytestmark = pytest.mark.gpu


def shard_for(cfg, **kw):
    shard = Shard([s.numel for s in cfg.params], [cfg.wd_of(s) for s in cfg.params], cfg.R, **kw)
    W.fill_state(shard, cfg)
    return shard


def hp_of(cfg, t):
    return hyper_pair(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, loss_scale=cfg.loss_scale, step=t)


class SampledOracle:
    """Oracle state for a strided sample of every tensor's elements (valid for element-independent Adam)."""

    def __init__(self, shard, cfg, stride):
        self.idx = []
        for s in cfg.params:
            n = s.numel
            ix = torch.arange(0, n, stride, device=shard.device)
            tail = torch.arange(max(0, n - 9), n, device=shard.device)
            self.idx.append(torch.unique(torch.cat([ix, tail])))
        self.w = [to_np_f32(shard.w_of(k)[ix]) for k, ix in enumerate(self.idx)]
        self.m = [to_np_f32(shard.m_of(k)[ix]) for k, ix in enumerate(self.idx)]
        self.v = [to_np_f32(shard.v_of(k)[ix]) for k, ix in enumerate(self.idx)]
        self.count = sum(int(ix.numel()) for ix in self.idx)

    def step(self, shard, cfg, ohp):
        ots = [oracle.OracleTensor(w=self.w[k], m=self.m[k], v=self.v[k],
                                   grads=[grad_to_np(shard, shard.grad_of(r, k)[ix]) for r in range(cfg.R)],
                                   weight_decay=shard.wds[k]) for k, ix in enumerate(self.idx)]
        flag = oracle.adam_step(ots, ohp, threads=THREADS)
        self.w = [t.w_out for t in ots]
        self.m = [t.m_out for t in ots]
        self.v = [t.v_out for t in ots]
        self.w16 = [t.w16_out for t in ots]
        return flag

    def compare(self, shard, label):
        for k, ix in enumerate(self.idx):
            for name, got, want in (("w", shard.w_of(k), self.w[k]), ("m", shard.m_of(k), self.m[k]), ("v", shard.v_of(k), self.v[k])):
                ratio, rel, cnt = state_error(to_np_f32(got[ix]), want)
                assert ratio <= 1.0, "%s: tensor %d %s off by %.3g x the bound (max rel %.3g)" % (label, k, name, ratio, rel)
            d = half_ulp_distance(to_np_bits(shard.w16_of(k)[ix]), self.w16[k])
            assert d.size == 0 or d.max() <= 1, "%s: tensor %d fp16 weights differ by %d ulp" % (label, k, d.max())


def test_config1_adam_flat_1m_three_steps_whole():
    cfg = W.config(1)
    shard = shard_for(cfg)
    ost = OracleState(shard, [0])
    hps = [hp_of(cfg, t) for t in (1, 2, 3)]
    rep = run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "config 1",
                    lambda i: W.fill_grads(shard, cfg, i + 1), expect_flags=[0, 0, 0])
    print("config 1 worst bound ratios per step:", [r[0] for r in rep])
    shard.destroy()


def test_config2_adam_bert_large_sampled_and_whole_tensors():
    cfg = W.config(2)
    shard = shard_for(cfg)
    samp = SampledOracle(shard, cfg, stride=61)
    names = [s.name for s in cfg.params]
    whole = [names.index(n) for n in ("emb.position", "emb.ln.gamma", "layer0.q.weight", "layer0.q.bias",
                                      "layer11.ffn_in.weight", "layer23.ffn_ln.beta", "mlm.decoder_bias", "nsp.weight", "nsp.bias")]
    ost = OracleState(shard, whole)
    ghp, ohp = hp_of(cfg, 1)
    W.fill_grads(shard, cfg, 1)
    assert all_inputs_finite(shard)
    oflag_s = samp.step(shard, cfg, ohp)
    ots = ost.tensors(shard)
    oflag_w = oracle.adam_step(ots, ohp, threads=THREADS)
    gflag = shard.step(cc.cc_fused_adam_step, ghp)
    torch.cuda.synchronize()
    assert gflag == oflag_s == oflag_w == 0
    ost.adopt(ots)
    compare_committed(shard, ost, "config 2 whole tensors")
    samp.compare(shard, "config 2 sample")
    print("config 2: %d sampled + %d whole-tensor elements checked" % (samp.count, sum(cfg.params[k].numel for k in whole)))
    # all elements: the unfused pipeline from the same inputs gives the same bits
    fused = [x[shard.cur].clone() for x in (shard.w, shard.m, shard.v)] + [shard.w16[shard.cur].view(torch.int16).clone()]
    shard.cur = 1 - shard.cur                    # back to the pre-step copy; the step is replayed unfused
    assert shard.step(cc.cc_unfused_adam_step, ghp) == 0
    torch.cuda.synchronize()
    now = [shard.w[shard.cur], shard.m[shard.cur], shard.v[shard.cur], shard.w16[shard.cur].view(torch.int16)]
    assert all(torch.equal(a, b) for a, b in zip(fused, now))
    shard.destroy()


def lamb_config(cfg, whole_names, label):
    shard = shard_for(cfg)
    names = [s.name for s in cfg.params]
    whole = [names.index(n) for n in whole_names]
    ost = OracleState(shard, whole)
    hps = [hp_of(cfg, t) for t in range(1, cfg.steps + 1)]

    def fill(i):
        W.fill_grads(shard, cfg, i + 1)
        assert all_inputs_finite(shard)
    rep = run_steps(shard, ost, cc.cc_fused_lamb_step, oracle.lamb_step, hps, label, fill,
                    expect_flags=[0] * cfg.steps, check_untouched=False)
    print(label, "worst bound ratios per step:", [r[0] for r in rep],
          "whole-tensor elements checked:", sum(cfg.params[k].numel for k in whole))
    # all elements: replay the last step through the unfused pipeline
    ghp = hps[-1][0]
    fused = [x[shard.cur].clone() for x in (shard.w, shard.m, shard.v)] + [shard.w16[shard.cur].view(torch.int16).clone()]
    shard.cur = 1 - shard.cur
    assert shard.step(cc.cc_unfused_lamb_step, ghp) == 0
    torch.cuda.synchronize()
    now = [shard.w[shard.cur], shard.m[shard.cur], shard.v[shard.cur], shard.w16[shard.cur].view(torch.int16)]
    assert all(torch.equal(a, b) for a, b in zip(fused, now))
    shard.destroy()


def test_config3_lamb_bert_large_whole_tensors():
    lamb_config(W.config(3), ("emb.position", "emb.type", "emb.ln.gamma", "emb.ln.beta", "layer0.q.weight", "layer0.q.bias",
                              "layer7.attn_ln.gamma", "layer11.ffn_in.weight", "layer11.ffn_in.bias", "layer23.ffn_out.weight",
                              "mlm.decoder_bias", "nsp.weight", "nsp.bias"), "config 3")


def test_config5_lamb_8p3b_shard_whole_slices():
    lamb_config(W.config(5), ("layer0.slice", "layer71.slice", "emb.slice"), "config 5")


def test_config4_adam_gpt2_xl_overflow_skip():
    cfg = W.config(4)
    shard = shard_for(cfg)
    names = [s.name for s in cfg.params]
    k_inf = names.index(W.CFG4_INF_TENSOR)
    whole = [k_inf, names.index("h0.ln_1.gamma"), names.index("h47.mlp.proj.bias"), names.index("ln_f.beta")]
    ost = OracleState(shard, whole)
    samp = SampledOracle(shard, cfg, stride=211)
    # calls 1, 2, 3 run as steps t = 1, 2, 2: the second call carries the planted +inf and is skipped
    steps = [1, 2, 2]
    expect = [0, 1, 0]
    for call, (t, want) in enumerate(zip(steps, expect), start=1):
        ghp, ohp = hp_of(cfg, t)
        W.fill_grads(shard, cfg, call)
        torch.cuda.synchronize()
        assert all_inputs_finite(shard) == (want == 0)
        ots = ost.tensors(shard)
        oflag = oracle.adam_step(ots, ohp, threads=THREADS)       # holds the tensor with the planted value
        assert oflag == want
        before = shard.cur
        pre = [x[shard.cur].clone() for x in (shard.w, shard.m, shard.v)] if want else None
        gflag = shard.step(cc.cc_fused_adam_step, ghp)
        torch.cuda.synchronize()
        assert gflag == want, "config 4 call %d: flag %d" % (call, gflag)
        ost.adopt(ots)
        if want:
            assert shard.cur == before
            assert all(torch.equal(a, x[shard.cur]) for a, x in zip(pre, (shard.w, shard.m, shard.v)))   # every element untouched
        else:
            assert samp.step(shard, cfg, ohp) == 0
            samp.compare(shard, "config 4 call %d sample" % call)
        compare_committed(shard, ost, "config 4 call %d whole tensors" % call)
    print("config 4: %d sampled elements per step" % samp.count)
    shard.destroy()


def test_config2_list_with_fp32_gradient_slices_sampled():
    """The Float 32 variant of the workload (paper, Section 6.1.1): same list, the R slices kept in fp32."""
    cfg = W.config(2)
    shard = shard_for(cfg, grad_dtype=torch.float32)
    samp = SampledOracle(shard, cfg, stride=97)
    for t in (1, 2):
        ghp, ohp = hp_of(cfg, t)
        W.fill_grads(shard, cfg, t)
        assert samp.step(shard, cfg, ohp) == 0
        assert shard.step(cc.cc_fused_adam_step, ghp) == 0
        torch.cuda.synchronize()
        samp.compare(shard, "config 2 fp32 slices step %d" % t)
    shard.destroy()
