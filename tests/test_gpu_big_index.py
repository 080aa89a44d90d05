"""A tensor of more than 2^31 elements: element indices above 2^31 and byte offsets above 2^33 must not wrap.

Adam is element-wise, so the oracle can be given slices of the tensor: the start, the places where a 32-bit element
index or a 32-bit byte offset would wrap (element 2^30 = byte 2^32 of an fp32 array, element 2^31 = byte 2^32 of an
fp16 array), and the ragged end.  In place with the per-element guard, so that one copy of the state (26 GB) is enough.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import hyper_pair, to_np_bits, to_np_f32
from util import half_ulp_distance, state_error

pytestmark = pytest.mark.gpu

NUMEL = (1 << 31) + 3 * 4096 + 5
SLICES = [(0, 10000), ((1 << 30) - 5000, (1 << 30) + 5000), ((1 << 31) - 5000, (1 << 31) + 5000), (NUMEL - 9000, NUMEL)]


@pytest.mark.parametrize("schedule", [cc.CC_SCHEDULE_AUTO, cc.CC_SCHEDULE_PER_CHUNK])
def test_adam_on_a_tensor_of_more_than_2_to_31_elements(schedule):
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * (1 << 30):
        pytest.skip("needs 60 GB of free device memory")
    R = 2
    shard = Shard([NUMEL], [0.01], R, chunk_elems=4096, in_place=True, schedule=schedule)
    want_sched = cc.CC_SCHEDULE_ORDERED if schedule == cc.CC_SCHEDULE_AUTO else cc.CC_SCHEDULE_PER_CHUNK
    assert cc.cc_plan_schedule(shard.plans[0])[0] == want_sched
    gen = torch.Generator(device=shard.device)
    gen.manual_seed(31)
    shard.w[0].normal_(0.0, 0.02, generator=gen)
    shard.m[0].normal_(0.0, 3e-3, generator=gen)
    shard.v[0].normal_(0.0, 1e-3, generator=gen)
    shard.v[0].square_()
    for g in shard.grads:
        g.normal_(0.0, 1e-2, generator=gen)
    a0, b0 = SLICES[2]
    shard.grad_of(1, 0).view(torch.int16)[a0 + 5003] = 0x7C00           # one inf just above element 2^31: guarded, flagged
    torch.cuda.synchronize()
    ghp, ohp = hyper_pair(step=3, skip_mode=1)
    ots = []
    for a, b in SLICES:
        ots.append(oracle.OracleTensor(w=to_np_f32(shard.w_of(0)[a:b]), m=to_np_f32(shard.m_of(0)[a:b]), v=to_np_f32(shard.v_of(0)[a:b]),
                                       grads=[to_np_bits(shard.grad_of(r, 0)[a:b]) for r in range(R)], weight_decay=0.01))
    oflag = oracle.adam_step(ots, ohp, threads=4)
    gflag = shard.step(cc.cc_fused_adam_step, ghp)
    torch.cuda.synchronize()
    assert gflag == oflag == 1
    for (a, b), t in zip(SLICES, ots):
        for name, got, want in (("w", shard.w_of(0)[a:b], t.w_out), ("m", shard.m_of(0)[a:b], t.m_out), ("v", shard.v_of(0)[a:b], t.v_out)):
            ratio, rel, cnt = state_error(to_np_f32(got), want)
            assert ratio <= 1.0, "slice [%d, %d) %s off by %.3g x the bound" % (a, b, name, ratio)
        d = half_ulp_distance(to_np_bits(shard.w16_of(0)[a:b]), t.w16_out)
        assert d.max() <= 1
    # the guarded element kept its state bit for bit, its neighbours moved
    k = a0 + 5003
    assert float(shard.w_of(0)[k]) == float(ots[2].w[5003]) and float(shard.w_of(0)[k + 1]) != float(ots[2].w[5004])
    shard.destroy()
