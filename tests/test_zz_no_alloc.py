"""cc_fused_adam_step_static (the entry point that allocates nothing) against cc_fused_adam_step on a single-tensor
plan: same kernel, so every output must agree bit for bit, on two calls in a row, the second on a smaller tensor, and on
more calls that change the grid size back and forth (the shared counting words must come out of every launch ready for
the next, whatever the sizes)."""
import ctypes as C

import pytest
import torch

from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd.shard import Shard
from parity import seeded_grads, seeded_state

pytestmark = pytest.mark.gpu


def one_tensor_of(shard, src):
    dst = 1 - src
    return cc.Tensor(numel=shard.numels[0], w_in=shard.w[src], m_in=shard.m[src], v_in=shard.v[src],
                     w_out=shard.w[dst], m_out=shard.m[dst], v_out=shard.v[dst], w16_out=shard.w16[dst],
                     grad=list(shard.grads), weight_decay=shard.wds[0])


def bits(shard, c):
    return [shard.w[c].view(torch.int32).clone(), shard.m[c].view(torch.int32).clone(), shard.v[c].view(torch.int32).clone(),
            shard.w16[c].view(torch.int16).clone()]


def run_pair(n, R, seed, hp, inject=None):
    """The same seeded step through the plan and through the static entry point; returns nothing, asserts equality."""
    a = Shard([n], [0.01], R, chunk_elems=1024, align_elems=8)
    b = Shard([n], [0.01], R, chunk_elems=1024, align_elems=8)
    for sh in (a, b):
        seeded_state(sh, seed)
        seeded_grads(sh, seed * 10, 1e-2)
        if inject is not None:
            sh.grads[inject[0]].view(torch.int16)[inject[1]] = 0x7C00
    a.run(cc.cc_fused_adam_step, hp)
    cc.cc_fused_adam_step_static(one_tensor_of(b, 0), R, hp, b.flag)
    torch.cuda.synchronize()
    assert int(a.flag.item()) == int(b.flag.item()) == (1 if inject is not None else 0)
    for x, y in zip(bits(a, 1), bits(b, 1)):
        assert torch.equal(x, y)
    for x, y in zip(bits(a, 0), bits(b, 0)):          # inputs untouched
        assert torch.equal(x, y)
    a.destroy(); b.destroy()


def test_static_entry_point_matches_the_plan_two_calls_the_second_smaller():
    run_pair((1 << 18) + 777, 4, 3, cc.Hyper(step=1))
    run_pair(5000, 4, 4, cc.Hyper(step=2))


def test_static_entry_point_grid_sizes_back_and_forth_and_overflow():
    for i, n in enumerate((64, 300000, 1, 1024 * 130, 70000, 1024 * 127 + 5, (1 << 20) + 3, 2048)):
        run_pair(n, 1 + (i % 3) * 3, 20 + i, cc.Hyper(step=1 + i % 3, adam_mode=i % 2))
    run_pair(90000, 8, 31, cc.Hyper(step=1), inject=(3, 4567))      # a planted +inf raises the flag on both paths
    run_pair(2048, 2, 32, cc.Hyper(step=1))                          # and the next call is clean again


def test_static_entry_point_rejects_what_it_cannot_do():
    sh = Shard([4096], [0.0], 2, chunk_elems=1024, align_elems=8)
    t = one_tensor_of(sh, 0)
    big = cc.Tensor(numel=(1 << 26) + 1, w_in=t.w_in, m_in=t.m_in, v_in=t.v_in, w_out=t.w_out, m_out=t.m_out, v_out=t.v_out,
                    w16_out=t.w16_out, grad=t.grad, weight_decay=0.0)
    with pytest.raises(cc.CcError) as e:
        cc.cc_fused_adam_step_static(big, 2, cc.Hyper(), sh.flag)
    assert e.value.code == cc.CC_ERR_ARG and "maximum" in cc.cc_last_error()
    with pytest.raises(cc.CcError) as e:
        cc.cc_fused_adam_step_static(t, 17, cc.Hyper(), sh.flag)
    assert e.value.code == cc.CC_ERR_ARG
    aliased = cc.Tensor(numel=4096, w_in=t.w_in, m_in=t.m_in, v_in=t.v_in, w_out=t.m_in, m_out=t.m_out, v_out=t.v_out,
                        w16_out=t.w16_out, grad=t.grad, weight_decay=0.0)
    with pytest.raises(cc.CcError) as e:
        cc.cc_fused_adam_step_static(aliased, 2, cc.Hyper(), sh.flag)
    assert e.value.code == cc.CC_ERR_ALIAS
    in_place = cc.Tensor(numel=4096, w_in=t.w_in, m_in=t.m_in, v_in=t.v_in, w_out=t.w_in, m_out=t.m_in, v_out=t.v_in,
                         w16_out=t.w16_out, grad=t.grad, weight_decay=0.0)
    with pytest.raises(cc.CcError) as e:
        cc.cc_fused_adam_step_static(in_place, 2, cc.Hyper(skip_mode=0), sh.flag)
    assert e.value.code == cc.CC_ERR_ALIAS
    sh.flag.fill_(7)
    empty = cc.Tensor(numel=0, w_in=0, m_in=0, v_in=0, w_out=0, m_out=0, v_out=0, w16_out=0, grad=[0, 0], weight_decay=0.0)
    cc.cc_fused_adam_step_static(empty, 2, cc.Hyper(), sh.flag)
    torch.cuda.synchronize()
    assert int(sh.flag.item()) == 0
    sh.destroy()


def test_static_entry_point_flag_over_many_launches_of_random_size():
    """The counting words are shared by every call on the GPU and are never reset from outside: 300 launches of random
    size, a third of them with an inf or NaN planted at a random place (first element, last element, anywhere, in any
    slice), must each report exactly their own flag, whatever ran before."""
    import random
    rng = random.Random(7)
    R, nmax = 3, 1 << 19
    sh = Shard([nmax], [0.0], R, chunk_elems=1024, align_elems=8)
    seeded_state(sh, 1)
    seeded_grads(sh, 10, 1e-2)
    clean = [g.clone() for g in sh.grads]
    wrong = []
    for i in range(300):
        n = rng.choice((1, 63, 64, 1023, 1024, 1025, 4096, 65 * 1024, 127 * 1024, 128 * 1024 + 1, rng.randrange(1, nmax + 1)))
        want = 0
        if rng.random() < 0.33:
            r, where = rng.randrange(R), rng.choice((0, n - 1, rng.randrange(n)))
            sh.grads[r].view(torch.int16)[where] = rng.choice((0x7C00, -1024, 0x7E00))      # +inf, -inf (0xFC00), NaN
            want = 1
        t = cc.Tensor(numel=n, w_in=sh.w[0], m_in=sh.m[0], v_in=sh.v[0], w_out=sh.w[1], m_out=sh.m[1], v_out=sh.v[1],
                      w16_out=sh.w16[1], grad=list(sh.grads), weight_decay=0.0)
        cc.cc_fused_adam_step_static(t, R, cc.Hyper(step=1), sh.flag)
        got = int(sh.flag.item())
        if got != want:
            wrong.append((i, n, want, got))
        if want:
            for g, c in zip(sh.grads, clean):
                g.copy_(c)
    assert not wrong, wrong[:10]
    sh.destroy()


def test_static_entry_point_under_graph_capture():
    """It allocates nothing, so the very first call may already sit inside a capture; every replay gives the eager result."""
    n, R = 200000, 4
    a = Shard([n], [0.01], R, chunk_elems=1024, align_elems=8)
    b = Shard([n], [0.01], R, chunk_elems=1024, align_elems=8)
    for sh in (a, b):
        seeded_state(sh, 9)
        seeded_grads(sh, 90, 1e-2)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cc.cc_fused_adam_step_static(one_tensor_of(b, 0), R, cc.Hyper(step=1), b.flag)
    for rep in range(3):
        if rep:
            for sh in (a, b):
                seeded_grads(sh, 90 + rep, 1e-2)
                if rep == 2:
                    sh.grads[1].view(torch.int16)[n - 1] = 0x7C00
        a.run(cc.cc_fused_adam_step, cc.Hyper(step=1))
        g.replay()
        torch.cuda.synchronize()
        assert int(a.flag.item()) == int(b.flag.item()) == (1 if rep == 2 else 0)
        for x, y in zip(bits(a, 1), bits(b, 1)):
            assert torch.equal(x, y)
    a.destroy(); b.destroy()
