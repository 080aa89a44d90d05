"""Seeded random sweep over list shapes, R, modes, hyper-parameters, gradient type, chunk size, schedule and
pipeline: every case is compared with the oracle element by element (same bar as the hand-picked cases)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import OracleState, hyper_pair, run_steps, seeded_grads, seeded_state

pytestmark = pytest.mark.gpu


def draw_case(rng):
    T = int(rng.integers(1, 9))
    kinds = rng.integers(0, 5, T)
    numels = []
    for k in kinds:
        if k == 0:
            numels.append(int(rng.integers(0, 9)))                       # empty and tiny
        elif k == 1:
            numels.append(int(rng.integers(9, 1100)))
        elif k == 2:
            numels.append(int(rng.choice([1024, 2048, 4096, 8192, 12288])))  # exact multiples
        elif k == 3:
            numels.append(int(rng.integers(1100, 30000)))
        else:
            numels.append(int(rng.integers(30000, 90000)))
    if sum(numels) == 0:
        numels[0] = 17
    lamb = bool(rng.integers(0, 2))
    case = dict(numels=numels, R=int(rng.integers(1, 17)), lamb=lamb,
                chunk=int(rng.choice([0, 1024, 2048, 4096, 8192])),
                unfused=bool(rng.integers(0, 2)), f32=bool(rng.integers(0, 3) == 0),
                gstd=float(rng.choice([3e-5, 1e-3, 1e-2, 0.3])),
                wds=[float(rng.choice([0.0, 0.01, 0.1])) for _ in numels],
                hp=dict(lr=float(rng.choice([1e-4, 1e-3, 2e-2])), beta1=float(rng.choice([0.0, 0.5, 0.9, 0.95])),
                        beta2=float(rng.choice([0.9, 0.98, 0.999])), eps=float(rng.choice([1e-8, 1e-6, 1e-3])),
                        loss_scale=float(rng.choice([1.0, 128.0, 65536.0, 3.0, 1000.0])),
                        grad_average=int(rng.integers(0, 2))))
    if not lamb:
        case["hp"]["adam_mode"] = int(rng.integers(0, 2))
        case["in_place"] = bool(rng.integers(0, 3) == 0)
        case["hp"]["skip_mode"] = 1 if case["in_place"] else int(rng.integers(0, 2))
    else:
        case["in_place"] = False
    return case


def run_case(seed, c, rng, same_start=False, steps=2, **shard_kw):
    shard = Shard(c["numels"], c["wds"], c["R"], chunk_elems=c["chunk"], in_place=c["in_place"], align_elems=8,
                  grad_dtype=torch.float32 if c["f32"] else torch.float16, **shard_kw)
    seeded_state(shard, seed)
    ost = OracleState(shard, range(len(c["numels"])))
    if c["lamb"]:
        gpu_fn, ofn = (cc.cc_unfused_lamb_step if c["unfused"] else cc.cc_fused_lamb_step), oracle.lamb_step
    else:
        gpu_fn, ofn = (cc.cc_unfused_adam_step if c["unfused"] else cc.cc_fused_adam_step), oracle.adam_step
    t0 = int(rng.integers(1, 2000))
    hps = [hyper_pair(step=t0 + i, **c["hp"]) for i in range(steps)]
    run_steps(shard, ost, gpu_fn, ofn, hps, "random case %d %r" % (seed, c),
              lambda i: seeded_grads(shard, seed * 10 + i, c["gstd"] * c["hp"]["loss_scale"] if c["hp"]["loss_scale"] <= 128 else c["gstd"]),
              same_start=same_start)
    shard.destroy()


@pytest.mark.parametrize("seed", range(40))
def test_random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    run_case(seed, draw_case(rng), rng)


@pytest.mark.parametrize("seed", range(40))
def test_random_case_ordered_schedule(seed):
    """The same kind of draw on 4096-element chunks under the ordered persistent schedule, with a random number of
    workgroups (1 .. more than there are chunks) and larger tensors, so that several blocks of the table are in play."""
    rng = np.random.default_rng(5000 + seed)
    c = draw_case(rng)
    c["chunk"] = 4096
    c["numels"] = [n * int(rng.choice([1, 1, 3, 8])) for n in c["numels"]]
    run_case(seed, c, rng, schedule=cc.CC_SCHEDULE_ORDERED, workgroups=int(rng.choice([1, 2, 3, 5, 8, 13, 32, 100, 0])))


@pytest.mark.parametrize("seed", range(30))
def test_random_case_written_through_stores(seed):
    """The same kind of draw on the 128-thread kernels under the two cache policies whose vector stores are written in
    assembly (chunks of 1024 or 2048 elements; small tests would otherwise all run under the non-temporal policy)."""
    rng = np.random.default_rng(9000 + seed)
    c = draw_case(rng)
    c["chunk"] = int(rng.choice([1024, 2048]))
    run_case(seed, c, rng, cache_policy=int(rng.choice([cc.CC_CACHE_RESIDENT, cc.CC_CACHE_WRITE_THROUGH])))


@pytest.mark.parametrize("seed", range(40, 130))
def test_random_case_step_by_step(seed):
    """Three steps per draw, each taken by the oracle from the state the GPU committed, so that every single step is
    compared from identical inputs (the tests above let both sides run on from their own results, which also lets the
    admissible error of one step move the next).  The three kinds of launch above take turns."""
    kind = seed % 3
    rng = np.random.default_rng((1000, 5000, 9000)[kind] + seed)
    c = draw_case(rng)
    kw = {}
    if kind == 1:
        c["chunk"] = 4096
        c["numels"] = [n * int(rng.choice([1, 1, 3, 8])) for n in c["numels"]]
        kw = dict(schedule=cc.CC_SCHEDULE_ORDERED, workgroups=int(rng.choice([1, 2, 3, 5, 8, 13, 32, 100, 0])))
    elif kind == 2:
        c["chunk"] = int(rng.choice([1024, 2048]))
        kw = dict(cache_policy=int(rng.choice([cc.CC_CACHE_RESIDENT, cc.CC_CACHE_WRITE_THROUGH])))
    run_case(seed, c, rng, same_start=True, steps=3, **kw)
