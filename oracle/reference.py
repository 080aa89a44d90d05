"""ctypes front end of oracle.c: builds it with gcc, marshals numpy arrays, loops over tensors.

The arithmetic lives in oracle.c.  This file only (i) compiles and loads it, (ii) hands each tensor's
arrays to the C routines, and (iii) applies the whole-step skip rule across tensors: if any tensor's
reduced gradient holds an inf or NaN, a step in skip mode 0 leaves every output at its pre-step value.

Test infrastructure only; never imported by the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "epilogue.c")]
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c into liboracle.so next to it (plain C, -O2, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or any(os.path.getmtime(_LIB) < os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", tmp] + _SRCS + ["-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_f32p = C.POINTER(C.c_float)
_u16p = C.POINTER(C.c_uint16)
_u16pp = C.POINTER(_u16p)
_vpp = C.POINTER(C.c_void_p)


def _load():
    global _lib
    if _lib is None:
        # ORACLE_SO points the loader at another build of oracle.c; the mutation test uses it to show
        # that the pins reject deliberately broken copies.  Nothing else sets it.
        lib = C.CDLL(os.environ.get("ORACLE_SO") or build())
        lib.oracle_half_to_double.restype = C.c_double
        lib.oracle_half_to_double.argtypes = [C.c_uint16]
        lib.oracle_float_to_half.restype = C.c_uint16
        lib.oracle_float_to_half.argtypes = [C.c_float]
        lib.oracle_grad_overflow.restype = C.c_int
        lib.oracle_grad_overflow.argtypes = [C.c_uint64, C.c_int, _vpp, C.c_int]
        lib.oracle_keep_tensor.restype = None
        lib.oracle_keep_tensor.argtypes = [C.c_uint64, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p, _u16p]
        common = [C.c_uint64, C.c_int, _vpp, C.c_int, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p, _u16p,
                  C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int, C.c_int]
        lib.oracle_adam_tensor.restype = None
        lib.oracle_adam_tensor.argtypes = common + [C.c_int, C.c_int]
        lib.oracle_lamb_tensor.restype = None
        lib.oracle_lamb_tensor.argtypes = common + [C.POINTER(C.c_double)]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        lib.oracle_dropout_word.restype = C.c_uint32
        lib.oracle_dropout_word.argtypes = [C.c_uint64, C.c_uint64]
        lib.oracle_dropout_threshold.restype = C.c_uint32
        lib.oracle_dropout_threshold.argtypes = [C.c_float]
        lib.oracle_double_to_half.restype = C.c_uint16
        lib.oracle_double_to_half.argtypes = [C.c_double]
        lib.oracle_mp_epilogue.restype = None
        lib.oracle_mp_epilogue.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int, _u16pp, _u16p, _u16p, _u16p,
                                           C.c_float, C.c_uint64, C.POINTER(C.c_uint8)]
        _lib = lib
    return _lib


@dataclass
class Hyper:
    """Step scalars, as the fp32/int32 values the GPU library's C interface carries."""
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-6
    loss_scale: float = 1.0
    step: int = 1            # 1-based
    grad_average: int = 0    # 0: sum of the R slices, 1: divide by R
    adam_mode: int = 1       # 1: decoupled decay, 0: L2
    skip_mode: int = 0       # 0: whole-step skip on overflow, 1: per-element guard


@dataclass
class OracleTensor:
    """One tensor of the slice: fp32 state; R gradient slices, all uint16 (fp16 bit patterns) or all float32."""
    w: np.ndarray
    m: np.ndarray
    v: np.ndarray
    grads: Sequence[np.ndarray]
    weight_decay: float = 0.0
    # outputs, filled by adam_step / lamb_step
    w_out: Optional[np.ndarray] = None
    m_out: Optional[np.ndarray] = None
    v_out: Optional[np.ndarray] = None
    w16_out: Optional[np.ndarray] = None
    norms: Optional[Tuple[float, float]] = None


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(_f32p)


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(_u16p)


def _gptrs(grads: Sequence[np.ndarray], n: int):
    """(array of R pointers, 1 if the slices are fp32 else 0)"""
    f32 = int(grads[0].dtype == np.float32)
    arr = (C.c_void_p * len(grads))()
    for r, g in enumerate(grads):
        assert g.dtype == (np.float32 if f32 else np.uint16) and g.flags.c_contiguous and g.size == n
        arr[r] = g.ctypes.data
    return arr, f32


def _alloc_outputs(t: OracleTensor):
    n = t.w.size
    t.w_out = np.empty(n, np.float32)
    t.m_out = np.empty(n, np.float32)
    t.v_out = np.empty(n, np.float32)
    t.w16_out = np.empty(n, np.uint16)


def half_to_double(bits: int) -> float:
    return _load().oracle_half_to_double(int(bits))


def float_to_half(x: float) -> int:
    return _load().oracle_float_to_half(float(np.float32(x)))


def grad_overflow(grads: Sequence[np.ndarray], sum_f16: bool = False) -> int:
    n = grads[0].size
    ptrs, f32 = _gptrs(grads, n)
    return int(_load().oracle_grad_overflow(n, len(grads), ptrs, 2 if (sum_f16 and not f32) else f32))


def _map(fn, tensors, threads):
    if threads <= 1 or len(tensors) <= 1:
        return [fn(t) for t in tensors]
    with ThreadPoolExecutor(max_workers=threads) as ex:   # the C calls release the GIL
        return list(ex.map(fn, tensors))


def _keep(t: OracleTensor):
    _load().oracle_keep_tensor(t.w.size, _f32(t.w), _f32(t.m), _f32(t.v),
                               _f32(t.w_out), _f32(t.m_out), _f32(t.v_out), _u16(t.w16_out))


def adam_step(tensors: List[OracleTensor], hp: Hyper, threads: int = 1, sum_f16: bool = False) -> int:
    """One Adam step over every tensor of the slice; fills *_out, returns the overflow flag.

    threads > 1 only spreads whole tensors over host threads; each tensor is still one sequential loop.
    sum_f16: the reduced gradient passes through fp16 before the optimizer (the unfused fp16 all-reduce baseline).
    """
    lib = _load()
    for t in tensors:
        _alloc_outputs(t)
    flag = int(any(_map(lambda t: grad_overflow(t.grads, sum_f16) if t.w.size else 0, tensors, threads)))
    if flag and hp.skip_mode == 0:
        _map(_keep, tensors, threads)
        return flag

    def one(t: OracleTensor):
        n = t.w.size
        ptrs, f32 = _gptrs(t.grads, n)
        if sum_f16:
            assert not f32, "the fp16 intermediate is defined for fp16 slices"
            f32 = 2
        lib.oracle_adam_tensor(n, len(t.grads), ptrs, f32, _f32(t.w), _f32(t.m), _f32(t.v),
                               _f32(t.w_out), _f32(t.m_out), _f32(t.v_out), _u16(t.w16_out),
                               hp.lr, hp.beta1, hp.beta2, hp.eps, t.weight_decay, hp.loss_scale,
                               hp.step, hp.grad_average, hp.adam_mode, int(hp.skip_mode == 1))
    _map(one, tensors, threads)
    return flag


def lamb_step(tensors: List[OracleTensor], hp: Hyper, threads: int = 1) -> int:
    """One LAMB step (one trust ratio per tensor); whole-step skip on overflow. Returns the flag."""
    lib = _load()
    if hp.skip_mode != 0 or hp.adam_mode != 1:
        raise ValueError("LAMB is defined here for whole-step skip and decoupled decay only")
    for t in tensors:
        _alloc_outputs(t)
    flag = int(any(_map(lambda t: grad_overflow(t.grads) if t.w.size else 0, tensors, threads)))
    if flag:
        _map(_keep, tensors, threads)
        return flag

    def one(t: OracleTensor):
        n = t.w.size
        norms = (C.c_double * 2)()
        ptrs, f32 = _gptrs(t.grads, n)
        lib.oracle_lamb_tensor(n, len(t.grads), ptrs, f32, _f32(t.w), _f32(t.m), _f32(t.v),
                               _f32(t.w_out), _f32(t.m_out), _f32(t.v_out), _u16(t.w16_out),
                               hp.lr, hp.beta1, hp.beta2, hp.eps, t.weight_decay, hp.loss_scale,
                               hp.step, hp.grad_average, norms)
        t.norms = (norms[0], norms[1])
    _map(one, tensors, threads)
    return flag


# ---- model-parallel epilogue (oracle/epilogue.c) ----

def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, out)
    return tuple(out)


def dropout_word(seed: int, index: int) -> int:
    return _load().oracle_dropout_word(seed, index)


def dropout_threshold(p: float) -> int:
    return _load().oracle_dropout_threshold(p)


def double_to_half(x: float) -> int:
    return _load().oracle_double_to_half(x)


def mp_epilogue(partials: Sequence[np.ndarray], bias: np.ndarray, residual: np.ndarray, first: int, p: float, seed: int):
    """out = Dropout(sum of the R partial outputs + bias, p) + residual on one slice; returns (out bits, kept mask)."""
    n = residual.size
    arr = (_u16p * len(partials))()
    for r, x in enumerate(partials):
        assert x.dtype == np.uint16 and x.flags.c_contiguous and x.size == n
        arr[r] = x.ctypes.data_as(_u16p)
    out = np.empty(n, np.uint16)
    kept = np.empty(n, np.uint8)
    _load().oracle_mp_epilogue(n, first, bias.size, len(partials), arr, _u16(bias), _u16(residual), _u16(out),
                               p, seed, kept.ctypes.data_as(C.POINTER(C.c_uint8)))
    return out, kept
