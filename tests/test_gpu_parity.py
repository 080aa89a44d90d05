"""Parity of the HIP path with the CPU oracle on small shapes (several chunks, ragged tails, odd lists).

Every case calls the library through its C ABI and compares element by element with oracle/ on the same
seeded bits: fp32 w, m, v within 2e-6 (relative, with the tensor's rms as floor), fp16 weights within one
fp16 ulp, overflow flag exactly.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import (OracleState, compare_committed, hyper_pair, run_steps, seeded_grads, seeded_state, to_np_bits,
                    to_np_f32)

pytestmark = pytest.mark.gpu

TINY = [1, 2, 7, 8, 9, 63, 64, 65, 1023, 1024, 1025, 4097]
ODD_LIST = [5000, 0, 1, 4096, 12289, 3, 8192, 777, 0, 20481]


def wds_for(numels, wd=0.01):
    return [wd if (i % 3) else 0.0 for i in range(len(numels))]


def adam_case(numels, R, steps=2, chunk=0, in_place=False, seed=1, gstd=1e-2, label="", grad_dtype=torch.float16, **hkw):
    shard = Shard(numels, wds_for(numels), R, chunk_elems=chunk, in_place=in_place, align_elems=8, grad_dtype=grad_dtype)
    seeded_state(shard, seed)
    ost = OracleState(shard, range(len(numels)))
    hps = [hyper_pair(step=t, **hkw) for t in range(1, steps + 1)]
    rep = run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, label or "adam",
                    lambda i: seeded_grads(shard, seed * 100 + i, gstd))
    shard.destroy()
    return rep


def lamb_case(numels, R, steps=2, chunk=0, seed=1, gstd=1e-2, label="", gpu_fn=None, grad_dtype=torch.float16, **hkw):
    shard = Shard(numels, wds_for(numels), R, chunk_elems=chunk, align_elems=8, grad_dtype=grad_dtype)
    seeded_state(shard, seed)
    ost = OracleState(shard, range(len(numels)))
    hps = [hyper_pair(step=t, **hkw) for t in range(1, steps + 1)]
    rep = run_steps(shard, ost, gpu_fn or cc.cc_fused_lamb_step, oracle.lamb_step, hps, label or "lamb",
                    lambda i: seeded_grads(shard, seed * 100 + i, gstd))
    shard.destroy()
    return rep


@pytest.mark.parametrize("R", [1, 2, 3, 4, 8, 16])
def test_adam_tiny_tensors_every_R(R):
    adam_case(TINY, R, steps=2, label="adam tiny R=%d" % R)


@pytest.mark.parametrize("R", [5, 6, 7, 9, 10, 11, 12, 13, 14, 15])
def test_adam_remaining_R(R):
    adam_case([4097, 9], R, steps=1, label="adam R=%d" % R)


@pytest.mark.parametrize("chunk", [1024, 4096, 16384])
def test_adam_odd_list_chunk_sizes(chunk):
    adam_case(ODD_LIST, 4, steps=3, chunk=chunk, label="adam odd list chunk=%d" % chunk)


@pytest.mark.parametrize("kw", [
    dict(adam_mode=0), dict(grad_average=1), dict(loss_scale=1024.0), dict(loss_scale=3.0, grad_average=1),
    dict(lr=3e-2, beta1=0.5, beta2=0.9, eps=1e-8), dict(beta1=0.0, beta2=0.0), dict(skip_mode=1),
])
def test_adam_modes(kw):
    adam_case([4097, 65, 20000], 3, steps=2, label="adam %s" % kw, **kw)


def test_adam_in_place_guard_mode():
    adam_case(ODD_LIST, 4, steps=2, in_place=True, skip_mode=1, label="adam in place")


def test_adam_subnormal_range_gradients_and_extreme_weights():
    """Gradients ~N(0, 1e-3) put ~5 % of the values in the fp16 subnormal range, N(0, 3e-5) most of them;
    weights span fp16 subnormal, normal and overflow."""
    numels = [30000, 4097]
    shard = Shard(numels, [0.01, 0.0], 8, align_elems=8)
    seeded_state(shard, 3)
    w = shard.w[shard.cur]
    n = w.numel()
    scale = torch.ones(n, device=w.device)
    scale[0:n:5] = 1e-4          # fp16 subnormal range
    scale[1:n:5] = 1e-7          # below half the smallest subnormal
    scale[2:n:5] = 3e6           # above the largest fp16 value
    w.mul_(scale)
    shard.w16[shard.cur].copy_(w)
    ost = OracleState(shard, range(2))
    hps = [hyper_pair(step=t) for t in (1, 2)]
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam subnormal",
              lambda i: seeded_grads(shard, 30 + i, 1e-3 if i == 0 else 3e-5))
    bits = to_np_bits(shard.w16_of(0))
    assert ((bits & 0x7C00) == 0).any() and ((bits & 0x7FFF) == 0x7C00).any()   # subnormals and infinities were emitted
    g = to_np_bits(shard.grad_of(0, 0))
    assert np.mean(((g & 0x7C00) == 0) & ((g & 0x3FF) != 0)) > 0.9                # the last inputs really were subnormal
    shard.destroy()


def _inject(shard, r, k, idx, bits):
    shard.grad_of(r, k).view(torch.int16)[idx] = int(np.array(bits, dtype=np.uint16).view(np.int16))


@pytest.mark.parametrize("bits", [0x7C00, 0xFC00, 0x7E00, 0xFFFF])
def test_adam_overflow_whole_step_skip(bits):
    numels = [5000, 12289, 64]
    shard = Shard(numels, wds_for(numels), 4, align_elems=8)
    seeded_state(shard, 5)
    ost = OracleState(shard, range(3))

    def fill(i):
        seeded_grads(shard, 50 + i, 1e-2)
        if i == 1:
            _inject(shard, 2, 1, 12288, bits)      # last element of a ragged tail
    # call 0 is step 1, call 1 overflows and is skipped, call 2 repeats step 2 with fresh gradients
    hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam skip", fill, expect_flags=[0, 1, 0])
    shard.destroy()


def test_adam_opposite_infinities_and_guard_mode():
    numels = [9000, 100]
    shard = Shard(numels, [0.01, 0.0], 4, in_place=True, align_elems=8)
    seeded_state(shard, 6)
    ost = OracleState(shard, range(2))

    def fill(i):
        seeded_grads(shard, 60 + i, 1e-2)
        if i == 0:
            _inject(shard, 0, 0, 4100, 0x7C00)
            _inject(shard, 3, 0, 4100, 0xFC00)     # +inf + -inf = NaN
            _inject(shard, 1, 1, 99, 0x7D55)       # a NaN in a scalar-tail element
    hps = [hyper_pair(step=1, skip_mode=1), hyper_pair(step=2, skip_mode=1)]
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam guard", fill, expect_flags=[1, 0])
    shard.destroy()


def test_large_finite_sum_does_not_flag():
    """16 slices of the largest fp16 value sum to ~1e6: finite in fp32, so no flag (and a huge but finite update)."""
    shard = Shard([2048], [0.0], 16, align_elems=8)
    seeded_state(shard, 7)
    ost = OracleState(shard, [0])

    def fill(i):
        for g in shard.grads:
            g.view(torch.int16).fill_(0x7BFF)
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, [hyper_pair(step=1)], "adam big", fill, expect_flags=[0])
    shard.destroy()


@pytest.mark.parametrize("R", [1, 4, 8])
def test_lamb_tiny_and_odd(R):
    lamb_case(TINY, R, steps=2, label="lamb tiny R=%d" % R)
    lamb_case(ODD_LIST, R, steps=2, chunk=1024, label="lamb odd R=%d" % R)


@pytest.mark.parametrize("kw", [dict(grad_average=1), dict(loss_scale=512.0), dict(lr=1e-2, beta1=0.8, beta2=0.99, eps=1e-8)])
def test_lamb_modes(kw):
    lamb_case([4097, 65, 50000], 3, steps=2, label="lamb %s" % kw, **kw)


def test_lamb_zero_weight_and_zero_update_tensors():
    """||w|| = 0 (fresh biases) and ||u|| = 0 (no gradient, no history, no decay) both give ratio 1."""
    numels = [3000, 3000, 5000]
    shard = Shard(numels, [0.0, 0.0, 0.01], 2, align_elems=8)
    seeded_state(shard, 8, with_history=False)
    shard.w_of(0).zero_()
    shard.w16_of(0).zero_()
    ost = OracleState(shard, range(3))

    def fill(i):
        seeded_grads(shard, 80 + i, 1e-2)
        for r in range(2):
            shard.grad_of(r, 1).zero_()
    run_steps(shard, ost, cc.cc_fused_lamb_step, oracle.lamb_step, [hyper_pair(step=1)], "lamb zero", fill)
    assert torch.equal(shard.w_of(1), torch.from_numpy(ost.w[1]).cuda())      # untouched tensor stays bit-exact
    shard.destroy()


def test_lamb_overflow_skips_phase_two():
    numels = [6000, 2000]
    shard = Shard(numels, [0.01, 0.0], 4, align_elems=8)
    seeded_state(shard, 9)
    ost = OracleState(shard, range(2))

    def fill(i):
        seeded_grads(shard, 90 + i, 1e-2)
        if i == 1:
            _inject(shard, 1, 1, 7, 0x7C00)
    hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
    run_steps(shard, ost, cc.cc_fused_lamb_step, oracle.lamb_step, hps, "lamb skip", fill, expect_flags=[0, 1, 0])
    shard.destroy()


def test_lamb_norms_match_oracle_and_phases_compose():
    numels = [20000, 4097, 1]
    shard = Shard(numels, [0.01, 0.0, 0.01], 4, chunk_elems=1024, align_elems=8)
    seeded_state(shard, 10)
    ost = OracleState(shard, range(3))
    seeded_grads(shard, 100, 1e-2)
    ghp, ohp = hyper_pair(step=3)
    ots = ost.tensors(shard)
    oracle.lamb_step(ots, ohp)
    cc.cc_fused_lamb_phase1(shard.plans[shard.cur], ghp, shard.flag)
    sums = cc.cc_lamb_norms_read(shard.plans[shard.cur], 3)
    for (sw, su), t in zip(sums, ots):
        assert np.sqrt(sw) == pytest.approx(t.norms[0], rel=1e-6)
        assert np.sqrt(su) == pytest.approx(t.norms[1], rel=1e-6)
    cc.cc_fused_lamb_phase2(shard.plans[shard.cur], ghp, shard.flag)
    torch.cuda.synchronize()
    assert int(shard.flag.item()) == 0
    shard.commit()
    ost.adopt(ots)
    compare_committed(shard, ost, "lamb phases")
    shard.destroy()


def _two_phase_lamb_step(plan, hp, flag, stream=None):
    cc.cc_fused_lamb_phase1(plan, hp, flag, stream)
    cc.cc_fused_lamb_phase2(plan, hp, flag, stream)


@pytest.mark.parametrize("numels", [[1 << 19, 300 * 1024 + 5, 0, 65 * 1024, 64 * 1024 + 1, 7], [512 * 1024 + 1, 3000]])
def test_lamb_step_call_and_its_two_phase_calls_give_the_same_bits(numels):
    """cc_fused_lamb_step lets the phase-2 workgroups add up their own tensor's partials when no tensor has more than
    512 chunks (first list: 512, 301, 0, 65, 65 and 1 chunks; second list: 513, the three-launch way); the two phase
    calls always launch the per-tensor kernel.  Sums and state must agree bit for bit, and with the oracle."""
    outs = []
    for fn in (cc.cc_fused_lamb_step, _two_phase_lamb_step):
        shard = Shard(numels, [0.01, 0.0, 0.01, 0.01, 0.0, 0.01][:len(numels)], 4, chunk_elems=1024, align_elems=8)
        seeded_state(shard, 21)
        ost = OracleState(shard, range(len(numels)))
        sums = []
        for t in (1, 2):
            seeded_grads(shard, 210 + t, 1e-2)
            ghp, ohp = hyper_pair(step=t)
            ots = ost.tensors(shard)
            oracle.lamb_step(ots, ohp)
            plan = shard.plans[shard.cur]
            shard.run(fn, ghp)
            got = cc.cc_lamb_norms_read(plan, len(numels))
            for (sw, su), o, n in zip(got, ots, numels):
                if n == 0:
                    assert sw == 0.0 and su == 0.0
                else:
                    assert np.sqrt(sw) == pytest.approx(o.norms[0], rel=1e-6) and np.sqrt(su) == pytest.approx(o.norms[1], rel=1e-6)
            sums.append(np.asarray(got))
            assert int(shard.flag.item()) == 0
            shard.commit()
            ost.adopt(ots)
            compare_committed(shard, ost, "lamb step %d" % t)
        outs.append((sums, shard.w[shard.cur].cpu(), shard.m[shard.cur].cpu(), shard.v[shard.cur].cpu(),
                     shard.w16[shard.cur].view(torch.int16).cpu()))
        shard.destroy()
    (sa, *a), (sb, *b) = outs
    assert all(np.array_equal(x.view(np.int64), y.view(np.int64)) for x, y in zip(sa, sb)), "the two ways add in different orders"
    assert _same(a, b)


# ---------------------------------------------------------------------------- invariances on the GPU side

def _gpu_adam_bits(numels, R, chunk, fn=None, flat=False, hkw=None, seed=11):
    """Runs two Adam steps and returns the concatenated committed state bits."""
    hkw = hkw or {}
    total = sum(numels)
    shard = Shard([total] if flat else numels, [0.01] if flat else [0.01] * len(numels), R, chunk_elems=chunk, align_elems=8)
    # identical logical content regardless of layout: generate flat, scatter into the tensors
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    w = torch.empty(total, device="cuda").normal_(0, 0.02, generator=g)
    m = torch.empty(total, device="cuda").normal_(0, 3e-3, generator=g)
    v = torch.empty(total, device="cuda").normal_(0, 1e-3, generator=g).square_()
    def scatter(dst_of, src):
        o = 0
        for k, n in enumerate(shard.numels):
            dst_of(k).copy_(src[o:o + n]); o += n
    scatter(shard.w_of, w); scatter(shard.m_of, m); scatter(shard.v_of, v)
    for t in (1, 2):
        for r in range(R):
            gr = torch.empty(total, device="cuda").normal_(0, 1e-2, generator=g).half()
            scatter(lambda k: shard.grad_of(r, k), gr)
        assert shard.step(fn or cc.cc_fused_adam_step, cc.Hyper(step=t, **hkw)) == 0
    torch.cuda.synchronize()
    cat = lambda of: torch.cat([of(k) for k in range(len(shard.numels))]).cpu()
    out = (cat(shard.w_of), cat(shard.m_of), cat(shard.v_of), cat(shard.w16_of).view(torch.int16))
    shard.destroy()
    return out


def _same(a, b):
    return all(torch.equal(x, y) for x, y in zip(a, b))


def test_adam_bits_do_not_depend_on_chunk_size_or_layout():
    numels = [5000, 1, 4096, 12289, 777, 20481]
    ref = _gpu_adam_bits(numels, 4, 4096)
    assert _same(ref, _gpu_adam_bits(numels, 4, 1024))
    assert _same(ref, _gpu_adam_bits(numels, 4, 32768))
    assert _same(ref, _gpu_adam_bits(numels, 4, 4096, flat=True))     # one contiguous tensor, same elements


@pytest.mark.parametrize("hkw", [dict(), dict(adam_mode=0), dict(loss_scale=64.0, grad_average=1)])
def test_fused_equals_unfused_adam_bit_for_bit(hkw):
    numels = [5000, 1, 4096, 12289, 777]
    assert _same(_gpu_adam_bits(numels, 8, 0, hkw=hkw), _gpu_adam_bits(numels, 8, 0, fn=cc.cc_unfused_adam_step, hkw=hkw))


def test_unfused_pipelines_against_oracle():
    numels = ODD_LIST
    shard = Shard(numels, wds_for(numels), 4, align_elems=8)
    seeded_state(shard, 12)
    ost = OracleState(shard, range(len(numels)))

    def fill(i):
        seeded_grads(shard, 120 + i, 1e-2)
        if i == 1:
            _inject(shard, 0, 4, 5, 0x7C00)
    hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
    run_steps(shard, ost, cc.cc_unfused_adam_step, oracle.adam_step, hps, "unfused adam", fill, expect_flags=[0, 1, 0])
    shard.destroy()
    lamb_case(ODD_LIST, 4, steps=2, label="unfused lamb", gpu_fn=cc.cc_unfused_lamb_step)


def test_fused_equals_unfused_lamb_bit_for_bit():
    def run(fn):
        numels = [5000, 4096, 12289, 3]
        shard = Shard(numels, [0.01] * 4, 4, align_elems=8)
        seeded_state(shard, 13)
        for t in (1, 2):
            seeded_grads(shard, 130 + t, 1e-2)
            assert shard.step(fn, cc.Hyper(step=t)) == 0
        torch.cuda.synchronize()
        out = (shard.w[shard.cur].cpu(), shard.m[shard.cur].cpu(), shard.v[shard.cur].cpu(),
               shard.w16[shard.cur].view(torch.int16).cpu())
        shard.destroy()
        return out
    assert _same(run(cc.cc_fused_lamb_step), run(cc.cc_unfused_lamb_step))


def test_lamb_is_deterministic_across_runs():
    def run():
        shard = Shard([300000, 4097], [0.01, 0.0], 8, align_elems=8)
        seeded_state(shard, 14)
        seeded_grads(shard, 140, 1e-3)
        assert shard.step(cc.cc_fused_lamb_step, cc.Hyper(step=1)) == 0
        torch.cuda.synchronize()
        out = (shard.w[shard.cur].cpu(), shard.m[shard.cur].cpu())
        shard.destroy()
        return out
    assert _same(run(), run())


def test_skewed_base_pointers():
    """Bases that are 16-byte but not 256-byte aligned."""
    numels = [4097, 8200, 33]
    shard = Shard(numels, wds_for(numels), 4, align_elems=8, skew_elems=8)
    seeded_state(shard, 15)
    ost = OracleState(shard, range(3))
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, [hyper_pair(step=1)], "adam skew",
              lambda i: seeded_grads(shard, 150, 1e-2))
    shard.destroy()


def test_state_copied_out_and_back_continues_identically():
    """The state is the caller's (w, m, v, step): restoring a copy of it resumes bit-identically."""
    def run(resume):
        shard = Shard([10000, 77], [0.01, 0.0], 4, align_elems=8)
        seeded_state(shard, 16)
        for t in (1, 2, 3):
            seeded_grads(shard, 160 + t, 1e-2)
            shard.step(cc.cc_fused_adam_step, cc.Hyper(step=t))
            if resume and t == 2:
                saved = [x[shard.cur].cpu() for x in (shard.w, shard.m, shard.v)]
                fresh = Shard([10000, 77], [0.01, 0.0], 4, align_elems=8)
                for dst, src in zip((fresh.w, fresh.m, fresh.v), saved):
                    dst[fresh.cur].copy_(src)
                shard.destroy()
                shard = fresh
        torch.cuda.synchronize()
        out = (shard.w[shard.cur].cpu(), shard.m[shard.cur].cpu(), shard.v[shard.cur].cpu())
        shard.destroy()
        return out
    assert _same(run(False), run(True))


# ---------------------------------------------------------------------------- fp32 gradient slices

@pytest.mark.parametrize("R", [1, 3, 8, 16])
def test_fp32_gradients_adam(R):
    adam_case(TINY + [20481], R, steps=2, grad_dtype=torch.float32, label="adam fp32 grads R=%d" % R)
    adam_case(ODD_LIST, R, steps=2, chunk=4096, grad_dtype=torch.float32, loss_scale=128.0, label="adam fp32 grads big chunk R=%d" % R)


@pytest.mark.parametrize("fn,ofn", [(cc.cc_fused_lamb_step, oracle.lamb_step), (cc.cc_unfused_lamb_step, oracle.lamb_step)])
def test_fp32_gradients_lamb(fn, ofn):
    lamb_case(ODD_LIST + [50000], 4, steps=2, grad_dtype=torch.float32, gpu_fn=fn, label="lamb fp32 grads")


def test_fp32_gradients_fused_equals_unfused_and_modes():
    def run(fn):
        numels = [5000, 4096, 12289, 3]
        shard = Shard(numels, [0.01] * 4, 8, align_elems=8, grad_dtype=torch.float32)
        seeded_state(shard, 17)
        for t in (1, 2):
            seeded_grads(shard, 170 + t, 1e-2)
            assert shard.step(fn, cc.Hyper(step=t, adam_mode=0, grad_average=1)) == 0
        torch.cuda.synchronize()
        out = (shard.w[shard.cur].cpu(), shard.m[shard.cur].cpu(), shard.v[shard.cur].cpu(),
               shard.w16[shard.cur].view(torch.int16).cpu())
        shard.destroy()
        return out
    assert _same(run(cc.cc_fused_adam_step), run(cc.cc_unfused_adam_step))
    adam_case([4097, 65], 3, steps=2, grad_dtype=torch.float32, adam_mode=0, grad_average=1, label="adam fp32 grads L2 avg")
    adam_case([4097, 65], 3, steps=2, grad_dtype=torch.float32, in_place=True, skip_mode=1, label="adam fp32 grads in place")


def test_fp32_gradients_overflow_cases():
    """inf and NaN inputs, and two finite slices whose fp32 sum overflows: all raise the flag and skip the step."""
    numels = [6000, 100]
    for case in ("inf", "nan", "finite overflow"):
        shard = Shard(numels, [0.01, 0.0], 2, align_elems=8, grad_dtype=torch.float32)
        seeded_state(shard, 18)
        ost = OracleState(shard, range(2))

        def fill(i):
            seeded_grads(shard, 180 + i, 1e-2)
            if i == 1:
                if case == "inf":
                    shard.grad_of(1, 0)[4099] = float("-inf")
                elif case == "nan":
                    shard.grad_of(0, 1)[99] = float("nan")
                else:
                    shard.grad_of(0, 0)[17] = 3e38
                    shard.grad_of(1, 0)[17] = 3e38
        hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
        run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam fp32 " + case, fill, expect_flags=[0, 1, 0])
        shard.destroy()


# ---------------------------------------------------------------------------- fp16 intermediate (the fp16 all-reduce baseline)

def _unfused_f16(plan, hp, flag, stream=None):
    cc.cc_unfused_adam_step_ex(plan, hp, flag, stream, cc.CC_GRAD_F16)


def _oracle_f16(tensors, hp, threads=1):
    return oracle.adam_step(tensors, hp, threads=threads, sum_f16=True)


@pytest.mark.parametrize("R,gstd", [(1, 1e-2), (8, 0.7), (16, 3.0)])
def test_unfused_adam_with_fp16_intermediate(R, gstd):
    numels = ODD_LIST + [40000]
    shard = Shard(numels, wds_for(numels), R, align_elems=8)
    seeded_state(shard, 19)
    ost = OracleState(shard, range(len(numels)))
    hps = [hyper_pair(step=t, loss_scale=4.0) for t in (1, 2)]
    run_steps(shard, ost, _unfused_f16, _oracle_f16, hps, "unfused fp16 intermediate R=%d" % R,
              lambda i: seeded_grads(shard, 190 + i, gstd))
    shard.destroy()


def test_fp16_intermediate_overflows_where_the_fused_sum_does_not():
    """Two slices of 60000 sum to 120000: finite in the fused kernel's fp32 registers, inf once it has to pass
    through fp16.  The baseline skips the step, the fused path takes it."""
    for fn, ofn, want in ((_unfused_f16, _oracle_f16, 1), (cc.cc_fused_adam_step, oracle.adam_step, 0)):
        shard = Shard([3000, 64], [0.01, 0.0], 2, align_elems=8)
        seeded_state(shard, 20)
        ost = OracleState(shard, range(2))

        def fill(i):
            seeded_grads(shard, 200 + i, 1e-2)
            for r in range(2):
                shard.grad_of(r, 1)[5] = 60000.0
        run_steps(shard, ost, fn, ofn, [hyper_pair(step=1, loss_scale=65536.0)], "fp16 range", fill, expect_flags=[want])
        shard.destroy()
    plan_f32 = Shard([64], [0.0], 2, align_elems=8, grad_dtype=torch.float32)
    with pytest.raises(cc.CcError) as e:
        _unfused_f16(plan_f32.plans[0], cc.Hyper(), plan_f32.flag)
    assert e.value.code == cc.CC_ERR_ARG
    plan_f32.destroy()


# ---- plans with one tensor: no table, descriptor in the kernel arguments ----

@pytest.mark.parametrize("numels", [[0, 5000, 0], [1], [1024], [1025], [4096 * 3], [4096 * 3 + 7], [0, 0, 20481]])
@pytest.mark.parametrize("chunk", [0, 4096])
def test_adam_single_tensor_plans(numels, chunk):
    adam_case(numels, 3, steps=2, chunk=chunk, label="adam single tensor %s chunk=%d" % (numels, chunk))


@pytest.mark.parametrize("kw", [dict(skip_mode=1), dict(adam_mode=0, grad_average=1)])
def test_adam_single_tensor_modes_and_fp32_gradients(kw):
    adam_case([0, 12289], 5, steps=2, label="adam single tensor %s" % kw, **kw)
    adam_case([12289], 2, steps=1, grad_dtype=torch.float32, label="adam single tensor fp32 %s" % kw, **kw)


def test_adam_single_tensor_overflow_skip():
    numels = [0, 9000]
    shard = Shard(numels, [0.0, 0.01], 4, align_elems=8)
    seeded_state(shard, 8)
    ost = OracleState(shard, range(2))

    def fill(i):
        seeded_grads(shard, 80 + i, 1e-2)
        if i == 1:
            _inject(shard, 3, 1, 8999, 0xFC00)
    hps = [hyper_pair(step=1), hyper_pair(step=2), hyper_pair(step=2)]
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam single tensor skip", fill, expect_flags=[0, 1, 0])
    shard.destroy()


@pytest.mark.parametrize("eps", [1e-8, 1e-3])
def test_adam_extreme_state_magnitudes(eps):
    """Second moments from 0 and 1e-30 up to 1e30 and first moments from 1e-20 to 1e18 against the oracle: the kernel
    forms the quotient from the hardware reciprocal and square root, which must hold the bound over the whole range.
    (Beyond ~1e36 the bias-corrected second moment v/(1 - beta2^t) leaves the fp32 range at small t, which fp32
    arithmetic cannot follow; the fp64 oracle can, so that corner is not compared.)  One second moment and one first
    moment per tensor, so that the rms floor of the bound is the magnitude under test."""
    vs = [0.0, 1e-30, 1e-10, 1.0, 1e20, 1e30]
    ms = [1e-20, -1e-20, 1.0, -1.0, 1e18, -1e18]
    cases = [(v, m) for v in vs for m in ms]
    numels = [300 + 7 * i for i in range(len(cases))]
    shard = Shard(numels, [0.01 if i % 2 else 0.0 for i in range(len(cases))], 2, align_elems=8)
    seeded_state(shard, 9)
    for k, (v, m) in enumerate(cases):
        shard.v_of(k).fill_(v)
        shard.m_of(k).fill_(m)
    ost = OracleState(shard, range(len(cases)))
    hps = [hyper_pair(step=t, eps=eps, beta2=0.98) for t in (1, 5)]
    run_steps(shard, ost, cc.cc_fused_adam_step, oracle.adam_step, hps, "adam extreme state eps=%g" % eps,
              lambda i: seeded_grads(shard, 90 + i, 1e-3))
    shard.destroy()
