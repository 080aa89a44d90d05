"""What a plan may vary without changing results: chunk size, cache policy; and what the unfused pipelines need first.

Adam is independent per element, so every chunk size and both cache policies must give the same bits.  LAMB adds its
per-chunk partial sums in double in a fixed order per chunk size; another chunk size groups them differently, so its
results move within rounding of the norms (checked against the oracle at the parity bar) while the cache policy leaves
the bits alone."""
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import OracleState, hyper_pair, run_steps, seeded_grads, seeded_state

pytestmark = pytest.mark.gpu

LIST = [16384 * 2 + 4097, 0, 1, 4096 * 3, 1024 * 9 + 1023, 8192, 777, 16384]


def wds_for(numels, wd=0.01):
    return [wd if (i % 3) else 0.0 for i in range(len(numels))]


def bits_of(sh):
    c = sh.cur
    return [sh.w[c].view(torch.int32).clone(), sh.m[c].view(torch.int32).clone(), sh.v[c].view(torch.int32).clone(),
            sh.w16[c].view(torch.int16).clone()]


def run_shape(fn, ofn, chunk, policy, R=4, grad_dtype=torch.float16, steps=2, numels=LIST):
    sh = Shard(numels, wds_for(numels), R, align_elems=8, grad_dtype=grad_dtype)
    for p in sh.plans:
        cc.cc_plan_set_chunk_elems(p, chunk)
        cc.cc_plan_set_cache_policy(p, policy)
        assert cc.cc_plan_layout(p)[0] == chunk
        want = policy if chunk < 4096 else cc.CC_CACHE_STREAMING
        assert cc.cc_plan_layout(p)[2] == want
    seeded_state(sh, 5)
    ost = OracleState(sh, range(len(numels)))
    run_steps(sh, ost, fn, ofn, [hyper_pair(step=t) for t in range(1, steps + 1)], "chunk %d policy %d" % (chunk, policy),
              lambda i: seeded_grads(sh, 500 + i, 1e-2), expect_flags=[0] * steps)
    out = bits_of(sh)
    sh.destroy()
    return out


@pytest.mark.parametrize("fn,ofn", [(cc.cc_fused_adam_step, oracle.adam_step), (cc.cc_unfused_adam_step, oracle.adam_step)])
def test_adam_bits_do_not_depend_on_chunk_size_or_cache_policy(fn, ofn):
    ref = run_shape(fn, ofn, 1024, cc.CC_CACHE_STREAMING)
    for chunk, policy in ((1024, cc.CC_CACHE_RESIDENT), (1024, cc.CC_CACHE_WRITE_THROUGH), (4096, cc.CC_CACHE_STREAMING),
                          (16384, cc.CC_CACHE_STREAMING), (4096, cc.CC_CACHE_RESIDENT)):
        got = run_shape(fn, ofn, chunk, policy)
        assert all(torch.equal(a, b) for a, b in zip(ref, got)), "chunk %d policy %d changes Adam's bits" % (chunk, policy)


@pytest.mark.parametrize("fn", [cc.cc_fused_lamb_step, cc.cc_unfused_lamb_step])
def test_lamb_every_chunk_size_and_policy_against_oracle(fn):
    per_chunk = {}
    for chunk, policy in ((1024, cc.CC_CACHE_STREAMING), (1024, cc.CC_CACHE_RESIDENT), (1024, cc.CC_CACHE_WRITE_THROUGH),
                          (4096, cc.CC_CACHE_STREAMING), (16384, cc.CC_CACHE_STREAMING)):
        got = run_shape(fn, oracle.lamb_step, chunk, policy)
        if chunk in per_chunk:          # same chunk size, other cache policy: the same bits
            assert all(torch.equal(a, b) for a, b in zip(per_chunk[chunk], got))
        per_chunk[chunk] = got


@pytest.mark.parametrize("R", [1, 8, 16])
def test_resident_policy_every_kind_of_R_and_fp32_slices(R):
    for gd in (torch.float16, torch.float32):
        a = run_shape(cc.cc_fused_adam_step, oracle.adam_step, 1024, cc.CC_CACHE_RESIDENT, R=R, grad_dtype=gd, steps=1)
        b = run_shape(cc.cc_fused_adam_step, oracle.adam_step, 1024, cc.CC_CACHE_STREAMING, R=R, grad_dtype=gd, steps=1)
        c = run_shape(cc.cc_fused_adam_step, oracle.adam_step, 1024, cc.CC_CACHE_WRITE_THROUGH, R=R, grad_dtype=gd, steps=1)
        assert all(torch.equal(x, y) and torch.equal(x, z) for x, y, z in zip(a, b, c))


def test_in_place_guard_mode_under_every_cache_policy():
    """skip_mode 1 reads and writes the same buffers; the written-through stores go through inline assembly, so the guard's
    "keep the input" case and the ordinary case are checked against the oracle under each policy, with an inf, a NaN made
    of opposite infinities and a NaN in a ragged tail planted in the first step, and the policies must agree bit for bit."""
    outs = []
    for policy in (cc.CC_CACHE_STREAMING, cc.CC_CACHE_RESIDENT, cc.CC_CACHE_WRITE_THROUGH):
        numels = [1024 * 9 + 1023, 100, 4096]
        sh = Shard(numels, [0.01, 0.0, 0.01], 4, in_place=True, align_elems=8, chunk_elems=1024, cache_policy=policy)
        assert cc.cc_plan_layout(sh.plans[0]) == (1024, 128, policy)
        seeded_state(sh, 6)
        ost = OracleState(sh, range(3))

        def fill(i):
            seeded_grads(sh, 60 + i, 1e-2)
            if i == 0:
                for r, t, e, bits in ((0, 0, 4100, 0x7C00), (3, 0, 4100, 0xFC00), (2, 0, 1024 * 9 + 1000, 0x7C00), (1, 1, 99, 0x7D55)):
                    sh.grad_of(r, t).view(torch.int16)[e] = bits - 0x10000 if bits >= 0x8000 else bits
        hps = [hyper_pair(step=1, skip_mode=1), hyper_pair(step=2, skip_mode=1), hyper_pair(step=3, skip_mode=1, adam_mode=0, grad_average=1)]
        run_steps(sh, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "guard, policy %d" % policy, fill, expect_flags=[1, 0, 0])
        outs.append(bits_of(sh))
        sh.destroy()
    for other in outs[1:]:
        assert all(torch.equal(a, b) for a, b in zip(outs[0], other))


def test_single_tensor_plan_resident_and_streaming():
    """One tensor: the table-free kernel, both policies, against the oracle (2^17 + a ragged end)."""
    for policy in (cc.CC_CACHE_RESIDENT, cc.CC_CACHE_STREAMING, cc.CC_CACHE_WRITE_THROUGH):
        run_shape(cc.cc_fused_adam_step, oracle.adam_step, 1024, policy, numels=[(1 << 17) + 5], steps=2)


def test_auto_policy_and_layout_rules():
    small = Shard([1 << 20], [0.0], 4, align_elems=8)                                  # 36 MB of buffers
    assert cc.cc_plan_layout(small.plans[0]) == (1024, 128, cc.CC_CACHE_RESIDENT)
    cc.cc_plan_set_cache_policy(small.plans[0], cc.CC_CACHE_STREAMING)
    assert cc.cc_plan_layout(small.plans[0])[2] == cc.CC_CACHE_STREAMING
    cc.cc_plan_set_cache_policy(small.plans[0], cc.CC_CACHE_RESIDENT)
    cc.cc_plan_set_chunk_elems(small.plans[0], 4096)
    assert cc.cc_plan_layout(small.plans[0]) == (4096, 512, cc.CC_CACHE_STREAMING)     # resident exists for 128-thread workgroups only
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_set_chunk_elems(small.plans[0], 2048)
    assert e.value.code == cc.CC_ERR_ARG
    with pytest.raises(cc.CcError):
        cc.cc_plan_set_cache_policy(small.plans[0], 9)
    cc.cc_plan_set_chunk_elems(small.plans[0], 0)
    assert cc.cc_plan_layout(small.plans[0]) == (1024, 128, cc.CC_CACHE_RESIDENT)
    cc.cc_plan_set_cache_policy(small.plans[0], cc.CC_CACHE_STREAMING)
    cc.cc_plan_set_cache_policy(small.plans[0], cc.CC_CACHE_AUTO)
    assert cc.cc_plan_layout(small.plans[0])[2] == cc.CC_CACHE_RESIDENT
    small.destroy()
    mid = Shard([1 << 22], [0.0], 8, align_elems=8, unfused=False)                      # 176 MB of buffers: still inside the Infinity Cache
    assert cc.cc_plan_layout(mid.plans[0]) == (1024, 128, cc.CC_CACHE_RESIDENT)
    mid.destroy()
    big = Shard([1 << 23], [0.0], 8, align_elems=8, unfused=False)                      # 352 MB: streams in, writes through
    assert cc.cc_plan_layout(big.plans[0]) == (1024, 128, cc.CC_CACHE_WRITE_THROUGH)
    big.destroy()
    tiny = Shard([1 << 16], [0.0], 8, align_elems=8, unfused=False)                     # 2.75 MB: launch-bound, streams
    assert cc.cc_plan_layout(tiny.plans[0]) == (1024, 128, cc.CC_CACHE_STREAMING)
    tiny.destroy()
    for mi, want in ((20, cc.CC_CACHE_WRITE_THROUGH), (21, cc.CC_CACHE_STREAMING)):     # 14 B stored per element against 288 MiB
        edge = Shard([mi << 20], [0.0], 2, align_elems=8, unfused=False)
        assert cc.cc_plan_layout(edge.plans[0]) == (1024, 128, want)
        edge.destroy()
    fixed = Shard([1 << 16], [0.0], 2, chunk_elems=2048, align_elems=8)                 # a caller's own chunk size: that one only
    assert cc.cc_plan_layout(fixed.plans[0])[:2] == (2048, 128)
    with pytest.raises(cc.CcError):
        cc.cc_plan_set_chunk_elems(fixed.plans[0], 4096)
    fixed.destroy()


def test_unfused_steps_need_the_reserved_buffer_and_never_allocate():
    sh = Shard([5000, 3], [0.01, 0.0], 2, align_elems=8, unfused=False)
    seeded_state(sh, 3)
    seeded_grads(sh, 30, 1e-2)
    before = bits_of(sh)
    for fn in (cc.cc_unfused_adam_step, cc.cc_unfused_lamb_step):
        with pytest.raises(cc.CcError) as e:
            sh.run(fn, cc.Hyper())
        assert e.value.code == cc.CC_ERR_ARG and "cc_plan_reserve_unfused" in cc.cc_last_error()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(before, bits_of(sh)))
    sh.reserve_unfused()
    sh.reserve_unfused()                                   # a second call does nothing
    # the very first unfused call can be captured into a graph: nothing is allocated or copied by a step call
    ref = Shard([5000, 3], [0.01, 0.0], 2, align_elems=8, unfused=True)
    seeded_state(ref, 3)
    seeded_grads(ref, 30, 1e-2)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sh.run(cc.cc_unfused_adam_step, cc.Hyper())
    g.replay()
    ref.run(cc.cc_unfused_adam_step, cc.Hyper())
    torch.cuda.synchronize()
    sh.commit(); ref.commit()
    assert all(torch.equal(a, b) for a, b in zip(bits_of(sh), bits_of(ref)))
    sh.destroy(); ref.destroy()


@pytest.mark.parametrize("log2n,R,policy", [(21, 8, cc.CC_CACHE_RESIDENT), (23, 2, cc.CC_CACHE_WRITE_THROUGH)])
@pytest.mark.parametrize("fn,ofn", [(cc.cc_fused_adam_step, oracle.adam_step), (cc.cc_fused_lamb_step, oracle.lamb_step)])
def test_mid_size_shard_under_the_automatic_cache_policy(fn, ofn, log2n, R, policy):
    """2^21 elements with R = 8 (88 MB of buffers: AUTO keeps the shard on chip) and 2^23 elements with R = 2 (252 MB, of
    which a launch stores 117 MB: AUTO writes through); two steps, every element against the oracle."""
    n = 1 << log2n
    sh = Shard([n - 4096 * 100 - 3, 4096 * 100 + 3], [0.01, 0.0], R, unfused=False)
    assert cc.cc_plan_layout(sh.plans[0]) == (1024, 128, policy)
    seeded_state(sh, 8)
    ost = OracleState(sh, [0, 1])
    run_steps(sh, ost, fn, ofn, [hyper_pair(step=t) for t in (1, 2)], "2^%d policy %d" % (log2n, policy),
              lambda i: seeded_grads(sh, 800 + i, 1e-3), expect_flags=[0, 0])
    sh.destroy()


@pytest.mark.parametrize("fn,ofn", [(cc.cc_fused_adam_step, oracle.adam_step), (cc.cc_fused_lamb_step, oracle.lamb_step),
                                    (cc.cc_unfused_adam_step, oracle.adam_step)])
def test_both_forms_of_the_chunk_table(fn, ofn):
    """Layouts of up to 2048 chunks give the kernels one copy of the tensor's descriptor per chunk, larger ones a chunk
    entry that points at the descriptor.  A list of exactly 2048 chunks and the same list with one more one-element
    tensor (2049 chunks) are each checked against the oracle, every element, two steps."""
    shared = [1024 * 700 + 5, 1024 * 1300, 17, 1024 * 44 + 1000, 1]            # 701 + 1300 + 1 + 45 + 1 = 2048 chunks
    for numels in (shared, shared + [1]):
        sh = Shard(numels, wds_for(numels), 3, align_elems=8, chunk_elems=1024, unfused=True)
        assert cc.cc_plan_info(sh.plans[0])[1] == len(numels) - 5 + 2048
        seeded_state(sh, 31)
        ost = OracleState(sh, range(len(numels)))
        run_steps(sh, ost, fn, ofn, [hyper_pair(step=t) for t in (1, 2)], "%d chunks" % (len(numels) - 5 + 2048),
                  lambda i: seeded_grads(sh, 310 + i, 1e-2), expect_flags=[0, 0])
        sh.destroy()
