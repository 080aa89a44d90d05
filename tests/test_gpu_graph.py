"""Step calls captured into a HIP graph: every replay must give what the same calls give eagerly.

The library clears nothing with memset nodes (the flag is written by the update kernel itself), so a captured
step is kernels only.  Replays are interleaved with eager work and synchronisation, and each one is checked."""
import pytest
import torch

from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import seeded_grads, seeded_state

pytestmark = pytest.mark.gpu


def _bits(shard):
    c = shard.cur
    # bit patterns, so that NaNs written by an overflowed step compare equal to themselves
    return [shard.w[c].view(torch.int32).clone(), shard.m[c].view(torch.int32).clone(), shard.v[c].view(torch.int32).clone(),
            shard.w16[c].view(torch.int16).clone(), shard.flag.clone()]


@pytest.mark.parametrize("schedule", [cc.CC_SCHEDULE_AUTO, cc.CC_SCHEDULE_ORDERED])
@pytest.mark.parametrize("fn", [cc.cc_fused_adam_step, cc.cc_fused_lamb_step, cc.cc_unfused_adam_step])
def test_graph_replays_match_eager(fn, schedule):
    """AUTO gives these small lists one workgroup per chunk; ORDERED forces the persistent schedule, whose work
    queue is handed back zeroed by the kernel itself (no memset node), with 7 workgroups for 82 chunks."""
    numels, wds, R = [20000, 4097, 3, 300000], [0.01, 0.0, 0.01, 0.01], 4
    kw = dict(chunk_elems=4096, schedule=schedule, workgroups=7) if schedule == cc.CC_SCHEDULE_ORDERED else {}
    eager = Shard(numels, wds, R, align_elems=8, **kw)
    graphed = Shard(numels, wds, R, align_elems=8, **kw)
    for s in (eager, graphed):
        seeded_state(s, 21)
        seeded_grads(s, 210, 1e-2)
    hps = [cc.Hyper(step=1), cc.Hyper(step=2)]

    def two_steps(s):                    # ping -> pong -> ping: the committed copy is the same buffer afterwards
        for hp in hps:
            s.run(fn, hp)
            s.commit()

    # warm up outside capture (module load, first-launch work), on a copy of the state that is then restored
    saved = [x.clone() for x in (graphed.w[0], graphed.m[0], graphed.v[0], graphed.w16[0])]
    two_steps(graphed)
    torch.cuda.synchronize()
    for dst, src in zip((graphed.w[0], graphed.m[0], graphed.v[0], graphed.w16[0]), saved):
        dst.copy_(src)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        two_steps(graphed)
    torch.cuda.synchronize()
    # capture records, it does not run: restore nothing, the state is still the seeded one
    for rep in range(4):
        if rep:                          # eager work between replays: fresh gradients for both shards
            for s in (eager, graphed):
                seeded_grads(s, 210 + rep, 1e-2)
            if rep == 2:                 # one replay with an overflow in its second step's inputs
                for s in (eager, graphed):
                    s.grad_of(1, 0).view(torch.int16)[17] = 0x7C00
            torch.cuda.synchronize()
        two_steps(eager)
        g.replay()
        torch.cuda.synchronize()
        a, b = _bits(eager), _bits(graphed)
        assert int(a[4].item()) == (1 if rep == 2 else 0)
        for x, y in zip(a, b):
            assert torch.equal(x, y), "replay %d differs from the eager run" % rep
    eager.destroy()
    graphed.destroy()
