"""The ordered persistent schedule (cc_plan_set_schedule) against the oracle and against one workgroup per chunk.

The schedule only changes which workgroup handles which chunk and when, so the fused Adam outputs must be
bit-identical between the two schedules, and so must LAMB's (its per-chunk partial sums are formed inside one
workgroup in a fixed order and added per tensor in a fixed order under both).  The lists mix many full chunks
with short last chunks and empty tensors, and the workgroup counts go from 1 (everything through one pipeline)
to more workgroups than chunks.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import OracleState, hyper_pair, run_steps, seeded_grads, seeded_state

pytestmark = pytest.mark.gpu

ORDERED = cc.CC_SCHEDULE_ORDERED
# 4096-element chunks: 4+1, 0, 1 short, 3 full, 9+1, 2 full, 1 short, 0, 30+1  (49 full + 5 short)
LIST = [4096 * 4 + 5, 0, 1, 4096 * 3, 4096 * 9 + 4095, 8192, 777, 0, 4096 * 30 + 1]
FULL_ONLY = [4096 * 7, 4096, 4096 * 12]
SHORT_ONLY = [5, 4095, 1, 100]


def wds_for(numels, wd=0.01):
    return [wd if (i % 3) else 0.0 for i in range(len(numels))]


def both_schedules(numels, R, gpu_fn, oracle_fn, workgroups, steps=2, seed=7, gstd=1e-2, grad_dtype=torch.float16,
                   in_place=False, inject=None, expect_flags=None, hps=None, **hkw):
    """Runs the same seeded steps under both schedules, checks the ordered one against the oracle and the two against
    each other bit for bit."""
    shards = []
    for sched, wgs in ((ORDERED, workgroups), (cc.CC_SCHEDULE_PER_CHUNK, 0)):
        sh = Shard(numels, wds_for(numels), R, chunk_elems=4096, align_elems=8, grad_dtype=grad_dtype, in_place=in_place,
                   schedule=sched, workgroups=wgs)
        assert cc.cc_plan_schedule(sh.plans[0])[0] == sched
        seeded_state(sh, seed)
        shards.append(sh)
    ordered, per_chunk = shards
    pairs = hps or [hyper_pair(step=t, **hkw) for t in range(1, steps + 1)]

    def fill_for(sh):
        def fill(i):
            seeded_grads(sh, seed * 100 + i, gstd)
            if inject is not None:
                inject(sh, i)
        return fill
    ost = OracleState(ordered, range(len(numels)))
    run_steps(ordered, ost, gpu_fn, oracle_fn, pairs, "ordered wgs=%d" % workgroups, fill_for(ordered), expect_flags=expect_flags)
    ost2 = OracleState(per_chunk, range(len(numels)))
    run_steps(per_chunk, ost2, gpu_fn, oracle_fn, pairs, "per chunk", fill_for(per_chunk), expect_flags=expect_flags)
    for k in range(len(numels)):
        for a, b in ((ordered.w_of(k), per_chunk.w_of(k)), (ordered.m_of(k), per_chunk.m_of(k)), (ordered.v_of(k), per_chunk.v_of(k))):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), "tensor %d differs between the schedules" % k
        assert torch.equal(ordered.w16_of(k).view(torch.int16), per_chunk.w16_of(k).view(torch.int16))
    for sh in shards:
        sh.destroy()


@pytest.mark.parametrize("workgroups", [1, 2, 3, 7, 24, 25, 64, 0])
def test_adam_ordered_workgroup_counts(workgroups):
    both_schedules(LIST, 4, cc.cc_fused_adam_step, oracle.adam_step, workgroups, steps=2)


@pytest.mark.parametrize("R", [1, 2, 3, 8, 13, 16])
def test_adam_ordered_every_kind_of_R(R):
    both_schedules(LIST, R, cc.cc_fused_adam_step, oracle.adam_step, 5, steps=1)


@pytest.mark.parametrize("numels", [FULL_ONLY, SHORT_ONLY, [4096], [4097], [1]])
@pytest.mark.parametrize("workgroups", [1, 3, 0])
def test_adam_ordered_degenerate_lists(numels, workgroups):
    both_schedules(numels, 3, cc.cc_fused_adam_step, oracle.adam_step, workgroups, steps=2)


@pytest.mark.parametrize("kw", [dict(adam_mode=0), dict(grad_average=1, loss_scale=8.0), dict(skip_mode=1)])
def test_adam_ordered_modes(kw):
    both_schedules(LIST, 3, cc.cc_fused_adam_step, oracle.adam_step, 6, steps=2, **kw)


def test_adam_ordered_in_place_guard():
    both_schedules(LIST, 4, cc.cc_fused_adam_step, oracle.adam_step, 6, steps=2, in_place=True, skip_mode=1)


@pytest.mark.parametrize("R", [2, 8, 12])
def test_adam_ordered_fp32_gradients(R):
    both_schedules(LIST, R, cc.cc_fused_adam_step, oracle.adam_step, 6, steps=1, grad_dtype=torch.float32)


def _inject_inf(where):
    def inject(sh, i):
        if i == 1:
            k, idx = where
            sh.grad_of(1, k).view(torch.int16)[idx] = int(np.array(0x7C00, dtype=np.uint16).view(np.int16))
    return inject


@pytest.mark.parametrize("where", [(0, 4096 * 4 + 4), (4, 17), (8, 4096 * 29 + 9)])
@pytest.mark.parametrize("fn", ["adam", "lamb"])
def test_ordered_overflow_skips_the_step(where, fn):
    """An inf in a short last chunk, in a tensor's first full chunk and in a late full chunk: flag 1, committed state
    untouched, and the repeated step matches the oracle."""
    gpu_fn, ofn = (cc.cc_fused_adam_step, oracle.adam_step) if fn == "adam" else (cc.cc_fused_lamb_step, oracle.lamb_step)
    hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
    both_schedules(LIST, 3, gpu_fn, ofn, 5, hps=hps, inject=_inject_inf(where), expect_flags=[0, 1, 0])


@pytest.mark.parametrize("workgroups", [1, 3, 24, 0])
def test_lamb_ordered(workgroups):
    both_schedules(LIST, 4, cc.cc_fused_lamb_step, oracle.lamb_step, workgroups, steps=2)


def test_lamb_ordered_fp32_gradients_and_many_slices():
    both_schedules(LIST, 8, cc.cc_fused_lamb_step, oracle.lamb_step, 6, steps=1, grad_dtype=torch.float32)
    both_schedules(FULL_ONLY + SHORT_ONLY, 16, cc.cc_fused_lamb_step, oracle.lamb_step, 4, steps=1)


@pytest.mark.parametrize("fn", ["adam", "adam16", "lamb"])
def test_unfused_pipelines_ordered(fn):
    if fn == "adam":
        both_schedules(LIST, 4, cc.cc_unfused_adam_step, oracle.adam_step, 5, steps=2)
    elif fn == "adam16":
        f = lambda plan, hp, flag, stream=None: cc.cc_unfused_adam_step_ex(plan, hp, flag, stream, cc.CC_GRAD_F16)
        o = lambda tensors, hp, threads=1: oracle.adam_step(tensors, hp, threads=threads, sum_f16=True)
        both_schedules(LIST, 4, f, o, 5, steps=2)
    else:
        both_schedules(LIST, 4, cc.cc_unfused_lamb_step, oracle.lamb_step, 5, steps=2)


def test_ordered_queue_is_clean_between_launches_and_kernels():
    """Adam, LAMB and the unfused pipelines share the plan's queue: alternate them many times on one plan and compare
    the final fused Adam step with a fresh plan's."""
    numels = LIST
    a = Shard(numels, wds_for(numels), 4, chunk_elems=4096, align_elems=8, schedule=ORDERED, workgroups=5)
    b = Shard(numels, wds_for(numels), 4, chunk_elems=4096, align_elems=8, schedule=ORDERED, workgroups=5)
    for sh in (a, b):
        seeded_state(sh, 11)
        seeded_grads(sh, 1100, 1e-2)
    ghp, _ = hyper_pair(step=1)
    for i, fn in enumerate((cc.cc_fused_lamb_step, cc.cc_unfused_adam_step, cc.cc_unfused_lamb_step, cc.cc_fused_adam_step) * 3):
        a.run(fn, ghp)          # writes the uncommitted copy only
        if i % 2 == 0:          # the ticket counter and the finished-workgroup word are zero after every step
            assert cc.cc_plan_queue_state(a.plans[a.cur]) == (0, 0)
    for _ in range(200):        # many launches back to back, then look once more
        a.run(cc.cc_fused_adam_step, ghp)
    assert cc.cc_plan_queue_state(a.plans[a.cur]) == (0, 0)
    a.run(cc.cc_fused_adam_step, ghp)
    b.run(cc.cc_fused_adam_step, ghp)
    torch.cuda.synchronize()
    assert int(a.flag.item()) == 0 and int(b.flag.item()) == 0
    a.commit(); b.commit()
    for k in range(len(numels)):
        assert torch.equal(a.w_of(k), b.w_of(k)) and torch.equal(a.m_of(k), b.m_of(k)) and torch.equal(a.v_of(k), b.v_of(k))
    a.destroy(); b.destroy()


def test_schedule_selection_and_errors():
    numels = [4096 * 3]
    sh = Shard(numels, [0.0], 2, chunk_elems=1024, align_elems=8)
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_set_schedule(sh.plans[0], ORDERED, 0)
    assert e.value.code == cc.CC_ERR_ARG
    with pytest.raises(cc.CcError):
        cc.cc_plan_set_schedule(sh.plans[0], 7, 0)
    with pytest.raises(cc.CcError):
        cc.cc_plan_set_schedule(sh.plans[0], cc.CC_SCHEDULE_AUTO, -1)
    assert cc.cc_plan_schedule(sh.plans[0])[0] == cc.CC_SCHEDULE_PER_CHUNK      # a small shard keeps one workgroup per chunk
    sh.destroy()
    sh = Shard(numels, [0.0], 2, chunk_elems=4096, align_elems=8)
    assert cc.cc_plan_schedule(sh.plans[0]) == (cc.CC_SCHEDULE_PER_CHUNK, 3)
    cc.cc_plan_set_schedule(sh.plans[0], ORDERED, 64)
    assert cc.cc_plan_schedule(sh.plans[0]) == (ORDERED, 2)                       # never more than pairs of chunks
    sh.destroy()


@pytest.mark.parametrize("optimizer", [0, 1])
def test_autotune_over_chunk_sizes_gives_the_oracle_result(optimizer):
    """A plan prepared for every chunk size: the tuner may land on any chunk size, schedule and cache policy; whatever it
    keeps, the steps that follow must agree with the oracle, and the trial steps must leave the committed copy alone."""
    numels = [4096 * 300 + 17, 4096 * 200, 5, 0, 16384 * 3 + 1]
    fn, ofn = (cc.cc_fused_adam_step, oracle.adam_step) if optimizer == 0 else (cc.cc_fused_lamb_step, oracle.lamb_step)
    tuned = Shard(numels, wds_for(numels), 4, align_elems=8)
    seeded_state(tuned, 19)
    seeded_grads(tuned, 1900, 1e-2)
    ghp, _ = hyper_pair(step=1)
    committed = [x.clone() for x in (tuned.w[0], tuned.m[0], tuned.v[0], tuned.w16[0])]
    # the trial steps of a plan write that plan's out buffers: tune the plan that reads the committed copy, then give the
    # other one (which writes the committed copy) the same shape by hand
    best_ms, per_chunk_ms = cc.cc_plan_autotune(tuned.plans[0], ghp, tuned.flag, optimizer)
    assert 0.0 < best_ms <= per_chunk_ms * 1.0001
    chunk, block, policy = cc.cc_plan_layout(tuned.plans[0])
    assert chunk in (1024, 4096, 16384) and block == (128 if chunk == 1024 else 512)
    assert policy in (cc.CC_CACHE_STREAMING, cc.CC_CACHE_RESIDENT, cc.CC_CACHE_WRITE_THROUGH)
    sched, wgs = cc.cc_plan_schedule(tuned.plans[0])
    assert sched in (cc.CC_SCHEDULE_PER_CHUNK, cc.CC_SCHEDULE_ORDERED) and wgs >= 1
    assert sched == cc.CC_SCHEDULE_PER_CHUNK or chunk == 4096
    cc.cc_plan_set_schedule(tuned.plans[1], cc.CC_SCHEDULE_PER_CHUNK, 0)
    cc.cc_plan_set_chunk_elems(tuned.plans[1], chunk)
    cc.cc_plan_set_schedule(tuned.plans[1], sched, wgs if sched == cc.CC_SCHEDULE_ORDERED else 0)
    cc.cc_plan_set_cache_policy(tuned.plans[1], policy)
    assert cc.cc_plan_layout(tuned.plans[1]) == (chunk, block, policy)
    for a, b in zip(committed, (tuned.w[0], tuned.m[0], tuned.v[0], tuned.w16[0])):
        assert torch.equal(a, b)
    ost = OracleState(tuned, range(len(numels)))
    run_steps(tuned, ost, fn, ofn, [hyper_pair(step=t) for t in (1, 2, 3)], "tuned plan", lambda i: seeded_grads(tuned, 1900 + i, 1e-2),
              expect_flags=[0, 0, 0])
    tuned.destroy()


@pytest.mark.parametrize("optimizer", [0, 1])
def test_autotune_keeps_a_valid_schedule_and_the_results(optimizer):
    numels = [4096 * 300 + 17, 4096 * 200, 5]
    fn = cc.cc_fused_adam_step if optimizer == 0 else cc.cc_fused_lamb_step
    tuned = Shard(numels, wds_for(numels), 4, chunk_elems=4096, align_elems=8)
    plain = Shard(numels, wds_for(numels), 4, chunk_elems=4096, align_elems=8, schedule=cc.CC_SCHEDULE_PER_CHUNK)
    for sh in (tuned, plain):
        seeded_state(sh, 17)
        seeded_grads(sh, 1700, 1e-2)
    ghp, _ = hyper_pair(step=2)
    committed = [x.clone() for x in (tuned.w[0], tuned.m[0], tuned.v[0], tuned.w16[0])]
    best_ms, per_chunk_ms = cc.cc_plan_autotune(tuned.plans[0], ghp, tuned.flag, optimizer)
    assert 0.0 < best_ms <= per_chunk_ms * 1.0001
    sched, wgs = cc.cc_plan_schedule(tuned.plans[0])
    assert sched in (cc.CC_SCHEDULE_PER_CHUNK, cc.CC_SCHEDULE_ORDERED) and wgs >= 1
    for a, b in zip(committed, (tuned.w[0], tuned.m[0], tuned.v[0], tuned.w16[0])):
        assert torch.equal(a, b)                                   # the trial steps left the committed copy alone
    assert tuned.step(fn, ghp) == 0 and plain.step(fn, ghp) == 0
    for k in range(len(numels)):
        assert torch.equal(tuned.w_of(k), plain.w_of(k)) and torch.equal(tuned.m_of(k), plain.m_of(k))
        assert torch.equal(tuned.v_of(k), plain.v_of(k)) and torch.equal(tuned.w16_of(k).view(torch.int16), plain.w16_of(k).view(torch.int16))
    tuned.destroy(); plain.destroy()


def test_autotune_rejects_in_place_plans_and_bad_arguments():
    sh = Shard([4096 * 4], [0.0], 2, chunk_elems=4096, align_elems=8, in_place=True)
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_autotune(sh.plans[0], cc.Hyper(skip_mode=1), sh.flag, 0)
    assert e.value.code == cc.CC_ERR_ALIAS
    sh.destroy()
    sh = Shard([4096 * 4], [0.0], 2, chunk_elems=4096, align_elems=8)
    before = cc.cc_plan_schedule(sh.plans[0])
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_autotune(sh.plans[0], cc.Hyper(), sh.flag, 2)
    assert e.value.code == cc.CC_ERR_ARG
    with pytest.raises(cc.CcError):
        cc.cc_plan_autotune(sh.plans[0], cc.Hyper(step=0), sh.flag, 0)
    assert cc.cc_plan_schedule(sh.plans[0]) == before
    sh.destroy()
