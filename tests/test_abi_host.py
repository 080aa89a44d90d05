"""Host-side checks that need no GPU: the library loads and exports what the header declares, the chunk table
is right, bad arguments are rejected before any device call, and the workload lists have the published sizes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2105_05720_amd import binding as cc
from paper_2105_05720_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ccfused.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = cc.load()
    names = declared_functions()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), "libccfused.so does not export %s" % n
        assert n in cc.EXPORTS, "binding does not type %s" % n
        assert hasattr(cc, n), "binding has no function %s" % n
    assert set(cc.EXPORTS) == set(names)
    assert cc.cc_version() == 200


def test_struct_layout_matches_header():
    assert C.sizeof(cc.cc_tensor) == 8 + 7 * 8 + 16 * 8 + 8      # numel, 7 pointers, 16 gradient pointers, float + pad
    assert cc.cc_tensor.weight_decay.offset == 192
    assert C.sizeof(cc.cc_hparams) == 36


def brute_table(numels, ce):
    out = []
    for t, n in enumerate(numels):
        for i in range(-(-n // ce)):
            out.append((t, i))
    return out


@pytest.mark.parametrize("ce", [1024, 4096, 8192])
def test_chunk_table_against_brute_force(ce):
    rng = np.random.default_rng(ce)
    numels = [0, 1, ce - 1, ce, ce + 1, 5 * ce, 0, 3] + [int(x) for x in rng.integers(0, 20 * ce, 20)]
    assert cc.cc_chunk_count(numels, ce) == len(brute_table(numels, ce))
    assert cc.cc_chunk_table_fill(numels, ce) == brute_table(numels, ce)
    # every element is covered exactly once and every chunk start is a multiple of 8 elements (16-byte accesses)
    covered = {t: 0 for t in range(len(numels))}
    for t, i in cc.cc_chunk_table_fill(numels, ce):
        assert (i * ce) % 8 == 0 and i * ce < numels[t]
        covered[t] += min(ce, numels[t] - i * ce)
    assert all(covered[t] == n for t, n in enumerate(numels))


@pytest.mark.parametrize("ce", [1024, 4096])
def test_ordered_table_against_brute_force(ce):
    """The ordered schedule's table: the same entries as the plain table, every full chunk first (tensor order),
    then the short last chunks; nfull counts the former."""
    rng = np.random.default_rng(ce + 1)
    numels = [0, 1, ce - 1, ce, ce + 1, 5 * ce, 0, 3, 7 * ce] + [int(x) for x in rng.integers(0, 20 * ce, 20)]
    plain = brute_table(numels, ce)
    full = [(t, i) for t, i in plain if (i + 1) * ce <= numels[t]]
    short = [(t, i) for t, i in plain if (i + 1) * ce > numels[t]]
    table, nfull = cc.cc_ordered_table_fill(numels, ce)
    assert nfull == len(full) == sum(n // ce for n in numels)
    assert table == full + short
    assert sorted(table) == sorted(plain) and len(short) == sum(1 for n in numels if n % ce)
    assert cc.cc_ordered_table_fill([], ce) == ([], 0)
    assert cc.cc_ordered_table_fill([ce * 3], ce) == ([(0, 0), (0, 1), (0, 2)], 3)
    assert cc.cc_ordered_table_fill([5], ce) == ([(0, 0)], 0)


def test_chunk_table_default_and_errors():
    assert cc.cc_default_chunk_elems() % 1024 == 0
    assert cc.cc_chunk_count([10000], 0) == -(-10000 // cc.cc_default_chunk_elems())
    assert cc.cc_chunk_count([], 1024) == 0
    for bad in (1000, -1024, 1):
        with pytest.raises(cc.CcError) as e:
            cc.cc_chunk_count([10], bad)
        assert e.value.code == cc.CC_ERR_ARG
    with pytest.raises(cc.CcError) as e:
        cc.cc_chunk_table_fill([5000, 5000], 1024, capacity=3)
    assert e.value.code == cc.CC_ERR_ARG and "capacity" in str(e.value)
    with pytest.raises(cc.CcError):
        cc.cc_chunk_count([2 ** 45], 1024)                      # would not fit one launch


def test_paper_bucket_table_accounting():
    """Section 5.4: 12 bytes per 2^10 elements; 0.6 % of a 334 M-element fp16 model."""
    enc_emb = sum(s.numel for s in W.bert_large_list() if not s.name.startswith(("pooler", "mlm", "nsp")))
    assert enc_emb == 334_092_288
    assert W.table_bytes_paper(enc_emb) == 12 * 326_262
    assert round(100 * W.table_bytes_paper(enc_emb) / (2 * enc_emb), 1) == 0.6
    assert W.table_bytes_paper(1) == 12 and W.table_bytes_paper(1025) == 24


def test_workload_sizes():
    want = {1: (1, 1_048_576), 2: (398, 336_226_108), 3: (398, 336_226_108), 4: (580, 1_557_611_200), 5: (73, 1_039_629_312)}
    for i, (T, N) in want.items():
        c = W.config(i)
        assert (len(c.params), c.numel) == (T, N)
    c4 = W.config(4)
    names = [s.name for s in c4.params]
    k = names.index(W.CFG4_INF_TENSOR)
    assert c4.params[k].numel == 1600 * 6400 and W.CFG4_INF_INDEX < c4.params[k].numel
    keys = {W.seed_key(s, t, r, k) for s in range(6) for t in range(4) for r in (0, 7, 99) for k in (0, 1, 579)}
    assert len(keys) == 6 * 4 * 3 * 3
    c2 = W.config(2)
    assert c2.wd_of(c2.params[0]) == 0.01 and c2.wd_of(c2.params[4]) == 0.0     # embedding decays, LayerNorm beta does not


def test_only_the_c_abi_is_exported():
    """The dynamic symbol table holds the declared entry points and nothing else (no kernel handles, no C++ helpers)."""
    import shutil
    import subprocess
    nm = shutil.which("nm")
    if nm is None:
        pytest.skip("nm is not installed")
    out = subprocess.check_output([nm, "-D", "--defined-only", cc.LIB_PATH], text=True)
    names = {line.split()[-1] for line in out.splitlines() if line.strip()}
    assert names == set(cc.EXPORTS), sorted(names ^ set(cc.EXPORTS))


def _tensor(**kw):
    base = dict(numel=4096, w_in=0x1000, m_in=0x10000, v_in=0x20000, w_out=0x30000, m_out=0x40000, v_out=0x50000,
                w16_out=0x60000, grad=[0x70000, 0x80000], weight_decay=0.0)
    base.update(kw)
    return cc.Tensor(**base)


@pytest.mark.parametrize("kw,R,code", [
    (dict(w_in=0), 2, cc.CC_ERR_NULL),
    (dict(w16_out=None), 2, cc.CC_ERR_NULL),
    (dict(grad=[0x70000, 0]), 2, cc.CC_ERR_NULL),
    (dict(m_in=0x10008), 2, cc.CC_ERR_ALIGN),
    (dict(grad=[0x70002, 0x80000]), 2, cc.CC_ERR_ALIGN),
    (dict(w_out=0x1000 + 64), 2, cc.CC_ERR_ALIAS),
    (dict(), 0, cc.CC_ERR_ARG),
    (dict(), 17, cc.CC_ERR_ARG),
    (dict(weight_decay=float("nan")), 2, cc.CC_ERR_ARG),
])
def test_plan_create_rejects_bad_arguments_on_the_host(kw, R, code):
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_create([_tensor(**kw)], R)
    assert e.value.code == code
    assert cc.cc_last_error()


# Overlap rules (checked on the host before any device call): an output buffer may share memory only with its own
# in-place input.  numel = 4096: fp32 buffers span 0x4000 bytes, fp16 ones 0x2000.
@pytest.mark.parametrize("tensors", [
    [dict(w16_out=0x30000 + 0x1000)],                                   # fp16 copy inside w_out
    [dict(grad=[0x40000 + 0x100, 0x80000])],                            # a gradient slice inside m_out
    [dict(v_in=0x30000)],                                               # v_in is w_out (not its own output)
    [dict(w_in=0x30000, w_out=0x30000, m_in=0x40000 + 16)],             # in place for w, m_in partially over m_out
    [dict(), dict(w_in=0x101000, m_in=0x110000, v_in=0x120000, w_out=0x50000 + 0x2000, m_out=0x140000, v_out=0x150000,
                  w16_out=0x160000, grad=[0x170000, 0x180000])],       # tensor 1's w_out inside tensor 0's v_out
    [dict(), dict(w_in=0x101000, m_in=0x110000, v_in=0x120000, w_out=0x130000, m_out=0x140000, v_out=0x150000,
                  w16_out=0x160000, grad=[0x60000, 0x180000])],        # tensor 1's gradient is tensor 0's fp16 output
    [dict(), dict(w_in=0x101000, m_in=0x110000, v_in=0x120000, w_out=0x130000, m_out=0x140000, v_out=0x150000,
                  w16_out=0x60000 + 0x1ff0, grad=[0x170000, 0x180000])],  # the two fp16 outputs share their last 16 bytes
])
def test_plan_create_rejects_overlaps_that_involve_an_output(tensors):
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_create([_tensor(**kw) for kw in tensors], 2)
    assert e.value.code == cc.CC_ERR_ALIAS
    assert "overlaps" in cc.cc_last_error()


@pytest.mark.parametrize("tensors", [
    [dict(grad=[0x70000, 0x70000])],                                    # the same slice twice: inputs may overlap inputs
    [dict(w_in=0x30000, w_out=0x30000, m_in=0x40000, m_out=0x40000, v_in=0x50000, v_out=0x50000)],   # in place
    [dict(w16_out=0x62000 - 0x2000)],                                   # buffers that touch end to start do not overlap
    [dict(), dict(numel=0, w_in=0, m_in=0, v_in=0, w_out=0, m_out=0, v_out=0, w16_out=0, grad=[0, 0])],   # empty tensors are not looked at
])
def test_plan_create_accepts_the_legal_sharing(tensors):
    # without a device the call gets past the host checks and then fails in the runtime; with one it succeeds
    try:
        plan = cc.cc_plan_create([_tensor(**kw) for kw in tensors], 2)
    except cc.CcError as e:
        assert e.code == cc.CC_ERR_HIP, cc.cc_last_error()
    else:
        plan.destroy()


def test_plan_create_rejects_empty_list_and_bad_chunk():
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_create([], 2)
    assert e.value.code == cc.CC_ERR_ARG
    with pytest.raises(cc.CcError) as e:
        cc.cc_plan_create([_tensor()], 2, chunk_elems=1000)
    assert e.value.code == cc.CC_ERR_ARG


def test_step_calls_reject_null_plan_and_bad_copy_arguments():
    lib = cc.load()
    hp = cc.Hyper().to_c()
    for name in ("cc_fused_adam_step", "cc_fused_lamb_step", "cc_unfused_adam_step", "cc_unfused_lamb_step",
                 "cc_fused_lamb_phase1", "cc_fused_lamb_phase2"):
        assert getattr(lib, name)(None, C.byref(hp), 0x1000, None) == cc.CC_ERR_NULL
    assert lib.cc_copy_probe(None, 0x1000, 16, None) == cc.CC_ERR_NULL
    assert lib.cc_copy_probe(0x1000, 0x2000, 17, None) == cc.CC_ERR_ARG
    assert lib.cc_copy_probe(0x1008, 0x2000, 32, None) == cc.CC_ERR_ALIGN
    assert lib.cc_plan_destroy(None) == cc.CC_OK
    assert lib.cc_plan_set_schedule(None, cc.CC_SCHEDULE_ORDERED, 0) == cc.CC_ERR_NULL
    assert lib.cc_plan_schedule(None, None, None) == cc.CC_ERR_NULL
    assert lib.cc_plan_autotune(None, C.byref(hp), 0, 0x1000, None, None, None) == cc.CC_ERR_NULL
    assert "plan is NULL" in cc.cc_last_error()
    assert lib.cc_plan_set_chunk_elems(None, 0) == cc.CC_ERR_NULL
    assert lib.cc_plan_layout(None, None, None, None) == cc.CC_ERR_NULL
    assert lib.cc_plan_set_cache_policy(None, 0) == cc.CC_ERR_NULL
    assert lib.cc_plan_reserve_unfused(None) == cc.CC_ERR_NULL
    assert lib.cc_plan_queue_state(None, None, None, None) == cc.CC_ERR_NULL
    assert lib.cc_pattern_probe(None, 4, 0, cc.CC_CACHE_STREAMING, 0x1000, None) == cc.CC_ERR_NULL
    t = cc._c_tensor(_tensor())
    assert lib.cc_pattern_probe(C.byref(t), 5, 0, cc.CC_CACHE_STREAMING, 0x1000, None) == cc.CC_ERR_ARG
    assert lib.cc_pattern_probe(C.byref(t), 4, 7, cc.CC_CACHE_STREAMING, 0x1000, None) == cc.CC_ERR_ARG
    t.numel = 1000
    assert lib.cc_pattern_probe(C.byref(t), 4, 1, cc.CC_CACHE_RESIDENT, 0x1000, None) == cc.CC_ERR_ARG
    assert "multiple of 1024" in cc.cc_last_error()


def test_static_step_rejects_bad_arguments_on_the_host():
    """The checks of the entry point that allocates nothing run before any device call."""
    lib = cc.load()
    hp = cc.Hyper().to_c()
    assert lib.cc_fused_adam_step_static(None, 2, C.byref(hp), 0x1000, None) == cc.CC_ERR_NULL

    def call(t, R=2, h=hp, flag=0x1000):
        c = cc._c_tensor(t)
        return lib.cc_fused_adam_step_static(C.byref(c), R, C.byref(h) if h is not None else None, flag, None)
    assert call(_tensor(), R=0) == cc.CC_ERR_ARG and call(_tensor(), R=17) == cc.CC_ERR_ARG
    assert call(_tensor(numel=(1 << 26) + 1)) == cc.CC_ERR_ARG and "maximum" in cc.cc_last_error()
    assert call(_tensor(w_in=0)) == cc.CC_ERR_NULL
    assert call(_tensor(grad=[0x70000, 0x80008])) == cc.CC_ERR_ALIGN
    assert call(_tensor(w16_out=0x30000 + 0x1000)) == cc.CC_ERR_ALIAS
    assert call(_tensor(grad=[0x40000 + 0x100, 0x80000])) == cc.CC_ERR_ALIAS
    assert call(_tensor(w_in=0x30000)) == cc.CC_ERR_ALIAS                       # in place needs skip_mode 1
    assert call(_tensor(), h=None) == cc.CC_ERR_NULL
    assert call(_tensor(), flag=None) == cc.CC_ERR_NULL
    assert call(_tensor(), h=cc.Hyper(step=0).to_c()) == cc.CC_ERR_ARG


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(cc, "_lib", None)
    monkeypatch.setattr(cc, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(FileNotFoundError):
        cc.cc_version()
