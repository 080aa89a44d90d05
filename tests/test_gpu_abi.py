"""Step-call argument checks that need a plan (hence a device): a rejected call enqueues nothing."""
import pytest
import torch

from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard

pytestmark = pytest.mark.gpu

STEPS = [cc.cc_fused_adam_step, cc.cc_unfused_adam_step, cc.cc_fused_lamb_step, cc.cc_unfused_lamb_step]


@pytest.mark.parametrize("kw,code", [
    (dict(step=0), cc.CC_ERR_ARG), (dict(step=-3), cc.CC_ERR_ARG),
    (dict(beta1=1.0), cc.CC_ERR_ARG), (dict(beta2=-0.1), cc.CC_ERR_ARG), (dict(beta1=float("nan")), cc.CC_ERR_ARG),
    (dict(loss_scale=0.0), cc.CC_ERR_ARG), (dict(loss_scale=float("inf")), cc.CC_ERR_ARG),
    (dict(loss_scale=float("nan")), cc.CC_ERR_ARG), (dict(eps=-1.0), cc.CC_ERR_ARG), (dict(lr=float("inf")), cc.CC_ERR_ARG),
    (dict(grad_average=2), cc.CC_ERR_ARG), (dict(adam_mode=5), cc.CC_ERR_ARG), (dict(skip_mode=2), cc.CC_ERR_ARG),
])
def test_bad_hyper_parameters_are_rejected_and_nothing_runs(kw, code):
    shard = Shard([5000], [0.01], 2, align_elems=8)
    shard.w[0].fill_(1.0)
    shard.flag.fill_(7)
    for fn in STEPS:
        with pytest.raises(cc.CcError) as e:
            fn(shard.plans[0], cc.Hyper(**kw), shard.flag)
        assert e.value.code == code
    torch.cuda.synchronize()
    assert int(shard.flag.item()) == 7                         # not even the flag was cleared
    assert float(shard.w[1].abs().max()) == 0.0                # and no output was written
    shard.destroy()


def test_null_flag_and_mode_restrictions():
    shard = Shard([5000], [0.01], 2, align_elems=8)
    for fn in STEPS:
        with pytest.raises(cc.CcError) as e:
            fn(shard.plans[0], cc.Hyper(), None)
        assert e.value.code == cc.CC_ERR_NULL
    for fn in (cc.cc_fused_lamb_step, cc.cc_unfused_lamb_step, cc.cc_fused_lamb_phase1, cc.cc_fused_lamb_phase2):
        for kw in (dict(skip_mode=1), dict(adam_mode=0)):
            with pytest.raises(cc.CcError) as e:
                fn(shard.plans[0], cc.Hyper(**kw), shard.flag)
            assert e.value.code == cc.CC_ERR_ARG
    shard.destroy()
    inplace = Shard([5000], [0.01], 2, in_place=True, align_elems=8)
    for fn in STEPS:
        with pytest.raises(cc.CcError) as e:
            fn(inplace.plans[0], cc.Hyper(skip_mode=0), inplace.flag)
        assert e.value.code == cc.CC_ERR_ALIAS
    inplace.destroy()


def test_plan_info_and_empty_tensors():
    shard = Shard([0, 5000, 0], [0.0, 0.01, 0.0], 3, chunk_elems=1024, align_elems=8)
    numel, chunks, table_bytes = cc.cc_plan_info(shard.plans[0])
    assert (numel, chunks) == (5000, 5) and table_bytes >= 5 * 8
    shard.flag.fill_(3)
    cc.cc_fused_adam_step(shard.plans[0], cc.Hyper(), shard.flag)
    torch.cuda.synchronize()
    assert int(shard.flag.item()) == 0
    shard.destroy()
    empty = Shard([0, 0], [0.0, 0.0], 1, align_elems=8)
    empty.flag.fill_(3)
    for fn in STEPS:
        fn(empty.plans[0], cc.Hyper(), empty.flag)
    torch.cuda.synchronize()
    assert int(empty.flag.item()) == 0
    empty.destroy()


def test_copy_probe_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    cc.cc_copy_probe(dst, src, src.numel() * 4 - 16)
    torch.cuda.synchronize()
    assert torch.equal(dst[:-4], src[:-4]) and int(dst[-4:].abs().sum()) == 0
