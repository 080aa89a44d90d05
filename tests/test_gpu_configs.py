"""The five benchmark configurations at full size, in the launch configuration bench.py times (default chunk size,
schedule and cache policy, out-of-place state), every element against the oracle.

The oracle keeps its own fp32 state of every tensor on the host and is fed the seeded gradients batch by batch; the
comparison (2e-6 relative on w, m, v with the rms floor, one fp16 ulp on the emitted weights, the flag bit for bit)
covers all N elements of every configuration, and for LAMB every tensor's pair of norms.  On top of that come the
properties that hold at any size: untouched inputs on a skipped step, and bit-equality of the fused result with the
unfused pipeline over all elements.
"""
import math

import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd import workloads as W
from paper_2105_05720_amd.shard import Shard
from parity import FullOracle, OracleState, all_inputs_finite, hyper_pair, run_steps

pytestmark = pytest.mark.gpu


def shard_for(cfg, **kw):
    shard = Shard([s.numel for s in cfg.params], [cfg.wd_of(s) for s in cfg.params], cfg.R, **kw)
    W.fill_state(shard, cfg)
    return shard


def hp_of(cfg, t):
    return hyper_pair(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, loss_scale=cfg.loss_scale, step=t)


def state_bits(shard):
    c = shard.cur
    return [shard.w[c].view(torch.int32).clone(), shard.m[c].view(torch.int32).clone(), shard.v[c].view(torch.int32).clone(),
            shard.w16[c].view(torch.int16).clone()]


def replay_unfused_and_compare(shard, unfused_fn, ghp, label):
    """The committed state came from a fused step; go back to the pre-step copy, run the unfused pipeline from the same
    inputs and require the same bits in every element."""
    fused = state_bits(shard)
    shard.reserve_unfused()
    shard.cur = 1 - shard.cur
    assert shard.step(unfused_fn, ghp) == 0
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(fused, state_bits(shard))), "%s: fused and unfused differ" % label


def test_config1_adam_flat_1m_three_steps_whole():
    cfg = W.config(1)
    shard = shard_for(cfg)
    assert cc.cc_plan_layout(shard.plans[0]) == (1024, 128, cc.CC_CACHE_RESIDENT)        # what bench.py times
    ost = OracleState(shard, [0])
    hps = [hp_of(cfg, t) for t in (1, 2, 3)]
    rep = run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "config 1",
                    lambda i: W.fill_grads(shard, cfg, i + 1), expect_flags=[0, 0, 0])
    print("config 1: %d of %d elements checked, worst bound ratios per step: %s" % (cfg.numel, cfg.numel, [r[0] for r in rep]))
    shard.destroy()


def check_lamb_norms(shard, full, label):
    """Every tensor's sum w^2 and sum u^2 as the kernels accumulated them against the oracle's norms."""
    got = cc.cc_lamb_norms_read(shard.plans[1 - shard.cur], len(shard.numels))     # the plan that ran the last committed step
    worst = 0.0
    for k, (sw, su) in enumerate(got):
        if shard.numels[k] == 0:
            continue
        nw, nu = full.norms[k]
        for a, b in ((math.sqrt(sw), nw), (math.sqrt(su), nu)):
            err = abs(a - b) / b if b > 0 else abs(a)
            worst = max(worst, err)
            assert err <= 1e-6, "%s: tensor %d norm %.9g, oracle %.9g" % (label, k, a, b)
    return worst


def full_size(index, unfused_fn):
    cfg = W.config(index)
    shard = shard_for(cfg)
    sched, wgs = cc.cc_plan_schedule(shard.plans[0])
    assert sched == cc.CC_SCHEDULE_ORDERED and wgs == cc.cc_device_info()[0]             # what bench.py times
    full = FullOracle(shard)
    fn = cc.cc_fused_adam_step if cfg.optimizer == "adam" else cc.cc_fused_lamb_step
    ghp = None
    for t in range(1, cfg.steps + 1):
        ghp, ohp = hp_of(cfg, t)
        W.fill_grads(shard, cfg, t)
        torch.cuda.synchronize()
        assert all_inputs_finite(shard)
        oflag = full.step(shard, ohp, cfg.optimizer)
        gflag = shard.step(fn, ghp)
        torch.cuda.synchronize()
        assert gflag == oflag == 0
        worst = full.compare(shard, "config %d step %d" % (index, t))
        line = "config %d step %d: %d of %d elements checked, worst %.3f x the bound" % (index, t, full.elements, cfg.numel, worst)
        if cfg.optimizer == "lamb":
            line += "; %d tensors' norms checked, worst relative error %.2e" % (len(cfg.params), check_lamb_norms(shard, full, "config %d" % index))
        print(line, flush=True)
    replay_unfused_and_compare(shard, unfused_fn, ghp, "config %d" % index)
    shard.destroy()


def test_config2_adam_bert_large_every_element():
    full_size(2, cc.cc_unfused_adam_step)


def test_config3_lamb_bert_large_every_element_and_every_norm():
    full_size(3, cc.cc_unfused_lamb_step)


def test_config5_lamb_8p3b_shard_every_element_and_every_norm():
    full_size(5, cc.cc_unfused_lamb_step)


def test_config4_adam_gpt2_xl_overflow_skip_every_element():
    cfg = W.config(4)
    shard = shard_for(cfg)
    assert cc.cc_plan_schedule(shard.plans[0])[0] == cc.CC_SCHEDULE_ORDERED
    full = FullOracle(shard)
    # calls 1, 2, 3 run as steps t = 1, 2, 2: the second call carries the planted +inf and is skipped
    ghp = None
    for call, (t, want) in enumerate(zip([1, 2, 2], [0, 1, 0]), start=1):
        ghp, ohp = hp_of(cfg, t)
        W.fill_grads(shard, cfg, call)
        torch.cuda.synchronize()
        assert all_inputs_finite(shard) == (want == 0)
        oflag = full.step(shard, ohp, "adam")
        assert oflag == want
        before = shard.cur
        pre = state_bits(shard) if want else None
        gflag = shard.step(cc.cc_fused_adam_step, ghp)
        torch.cuda.synchronize()
        assert gflag == want, "config 4 call %d: flag %d" % (call, gflag)
        if want:
            assert shard.cur == before
            assert all(torch.equal(a, b) for a, b in zip(pre, state_bits(shard)))        # every element untouched
        worst = full.compare(shard, "config 4 call %d" % call)
        print("config 4 call %d (flag %d): %d of %d elements checked, worst %.3f x the bound" % (call, want, full.elements, cfg.numel, worst), flush=True)
    replay_unfused_and_compare(shard, cc.cc_unfused_adam_step, ghp, "config 4")
    shard.destroy()


def test_config2_list_with_fp32_gradient_slices_every_element():
    """The Float 32 variant of the workload (paper, Section 6.1.1): same list, the R slices kept in fp32, under the
    schedule AUTO picks for it (ordered), two steps, every element."""
    cfg = W.config(2)
    shard = shard_for(cfg, grad_dtype=torch.float32)
    assert cc.cc_plan_schedule(shard.plans[0])[0] == cc.CC_SCHEDULE_ORDERED
    full = FullOracle(shard)
    for t in (1, 2):
        ghp, ohp = hp_of(cfg, t)
        W.fill_grads(shard, cfg, t)
        torch.cuda.synchronize()
        assert full.step(shard, ohp, "adam") == 0
        assert shard.step(cc.cc_fused_adam_step, ghp) == 0
        torch.cuda.synchronize()
        worst = full.compare(shard, "config 2 fp32 slices step %d" % t)
        print("config 2 with fp32 slices step %d: %d of %d elements checked, worst %.3f x the bound" % (t, full.elements, cfg.numel, worst), flush=True)
    shard.destroy()
