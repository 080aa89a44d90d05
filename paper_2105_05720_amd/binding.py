"""Thin ctypes layer over libccfused.so: same names as include/ccfused.h, argument marshalling only.

Device buffers are torch tensors (or raw integer device addresses); every step of the update runs in the
library's kernels.  The library is loaded on first use and a missing build raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

CC_MAX_R = 16
CC_GRAD_F16, CC_GRAD_F32 = 0, 1
CC_SCHEDULE_AUTO, CC_SCHEDULE_PER_CHUNK, CC_SCHEDULE_ORDERED = 0, 1, 2
CC_CACHE_AUTO, CC_CACHE_STREAMING, CC_CACHE_RESIDENT, CC_CACHE_WRITE_THROUGH = 0, 1, 2, 3
CC_OK, CC_ERR_NULL, CC_ERR_ARG, CC_ERR_ALIGN, CC_ERR_ALIAS, CC_ERR_HIP, CC_ERR_NOMEM = 0, -1, -2, -3, -4, -5, -6

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libccfused.so")
_lib = None


class CcError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("ccfused error %d: %s" % (code, message))
        self.code = code


class cc_tensor(C.Structure):
    _fields_ = [("numel", C.c_uint64),
                ("w_in", C.c_void_p), ("m_in", C.c_void_p), ("v_in", C.c_void_p),
                ("w_out", C.c_void_p), ("m_out", C.c_void_p), ("v_out", C.c_void_p),
                ("w16_out", C.c_void_p),
                ("grad", C.c_void_p * CC_MAX_R),
                ("weight_decay", C.c_float)]


class cc_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("loss_scale", C.c_float), ("step", C.c_int32), ("grad_average", C.c_int32),
                ("adam_mode", C.c_int32), ("skip_mode", C.c_int32)]


class cc_epilogue(C.Structure):
    _fields_ = [("numel", C.c_uint64), ("first", C.c_uint64), ("hidden", C.c_uint32), ("R", C.c_int32),
                ("partial", C.c_void_p * CC_MAX_R), ("bias", C.c_void_p), ("residual", C.c_void_p), ("out", C.c_void_p),
                ("dropout_p", C.c_float), ("seed", C.c_uint64)]


# every symbol include/ccfused.h declares
EXPORTS = {
    "cc_chunk_count": (C.c_int64, [C.POINTER(C.c_uint64), C.c_int32, C.c_int32]),
    "cc_chunk_table_fill": (C.c_int64, [C.POINTER(C.c_uint64), C.c_int32, C.c_int32, C.POINTER(C.c_uint32), C.c_int64]),
    "cc_ordered_table_fill": (C.c_int64, [C.POINTER(C.c_uint64), C.c_int32, C.c_int32, C.POINTER(C.c_uint32), C.c_int64,
                                          C.POINTER(C.c_int64)]),
    "cc_default_chunk_elems": (C.c_int32, []),
    "cc_plan_create": (C.c_int, [C.POINTER(cc_tensor), C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]),
    "cc_plan_create_ex": (C.c_int, [C.POINTER(cc_tensor), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]),
    "cc_plan_destroy": (C.c_int, [C.c_void_p]),
    "cc_plan_set_schedule": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "cc_plan_schedule": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "cc_plan_set_chunk_elems": (C.c_int, [C.c_void_p, C.c_int32]),
    "cc_plan_layout": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "cc_plan_set_cache_policy": (C.c_int, [C.c_void_p, C.c_int32]),
    "cc_plan_reserve_unfused": (C.c_int, [C.c_void_p]),
    "cc_plan_queue_state": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_uint64), C.c_void_p]),
    "cc_plan_autotune": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_int32, C.c_void_p, C.c_void_p,
                                   C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "cc_plan_info": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_int64), C.POINTER(C.c_uint64)]),
    "cc_fused_adam_step": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_fused_adam_step_static": (C.c_int, [C.POINTER(cc_tensor), C.c_int32, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_fused_lamb_step": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_fused_lamb_phase1": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_fused_lamb_phase2": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_lamb_norm_buffer": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p)]),
    "cc_lamb_norms_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.c_void_p]),
    "cc_unfused_adam_step": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_unfused_adam_step_ex": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p, C.c_int32]),
    "cc_unfused_lamb_step": (C.c_int, [C.c_void_p, C.POINTER(cc_hparams), C.c_void_p, C.c_void_p]),
    "cc_fused_epilogue": (C.c_int, [C.POINTER(cc_epilogue), C.c_void_p]),
    "cc_unfused_epilogue": (C.c_int, [C.POINTER(cc_epilogue), C.c_void_p, C.c_void_p]),
    "cc_pattern_probe": (C.c_int, [C.POINTER(cc_tensor), C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "cc_copy_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "cc_device_info": (C.c_int, [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]),
    "cc_last_error": (C.c_char_p, []),
    "cc_version": (C.c_int, []),
}


def load():
    """Loads libccfused.so (built by paper_2105_05720_amd.build) and types its entry points."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2105_05720_amd.build` (there is no CPU fallback)" % LIB_PATH)
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)          # AttributeError if the library does not export it
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise CcError(int(rc), load().cc_last_error().decode())
    return rc


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream or None
    return int(stream) or None


@dataclass
class Tensor:
    """Python-side spelling of cc_tensor: torch tensors or integer device addresses."""
    numel: int
    w_in: object
    m_in: object
    v_in: object
    w_out: object
    m_out: object
    v_out: object
    w16_out: object
    grad: Sequence[object]
    weight_decay: float = 0.0


@dataclass
class Hyper:
    """Python-side spelling of cc_hparams."""
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-6
    loss_scale: float = 1.0
    step: int = 1
    grad_average: int = 0
    adam_mode: int = 1
    skip_mode: int = 0

    def to_c(self) -> cc_hparams:
        return cc_hparams(self.lr, self.beta1, self.beta2, self.eps, self.loss_scale, self.step,
                          self.grad_average, self.adam_mode, self.skip_mode)


def _hp(hp) -> cc_hparams:
    return hp if isinstance(hp, cc_hparams) else hp.to_c()


class Plan:
    """Owns a cc_plan handle and keeps the buffers it points at alive."""

    def __init__(self, handle: int, keep):
        self.handle = handle
        self._keep = keep

    def destroy(self):
        if self.handle:
            load().cc_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---- host helpers of the chunk table ----

def cc_default_chunk_elems() -> int:
    return load().cc_default_chunk_elems()


def cc_chunk_count(numels: Sequence[int], chunk_elems: int = 0) -> int:
    arr = (C.c_uint64 * max(len(numels), 1))(*numels)
    return _check(load().cc_chunk_count(arr, len(numels), chunk_elems))


def cc_chunk_table_fill(numels: Sequence[int], chunk_elems: int = 0, capacity: Optional[int] = None):
    n = cc_chunk_count(numels, chunk_elems) if capacity is None else capacity
    arr = (C.c_uint64 * max(len(numels), 1))(*numels)
    table = (C.c_uint32 * max(2 * n, 2))()
    k = _check(load().cc_chunk_table_fill(arr, len(numels), chunk_elems, table, n))
    return [(table[2 * i], table[2 * i + 1]) for i in range(k)]


def cc_ordered_table_fill(numels: Sequence[int], chunk_elems: int = 0):
    """([(tensor, chunk)] in the ordered schedule's order, number of full chunks)."""
    n = cc_chunk_count(numels, chunk_elems)
    arr = (C.c_uint64 * max(len(numels), 1))(*numels)
    table = (C.c_uint32 * max(2 * n, 2))()
    nfull = C.c_int64()
    k = _check(load().cc_ordered_table_fill(arr, len(numels), chunk_elems, table, n, C.byref(nfull)))
    return [(table[2 * i], table[2 * i + 1]) for i in range(k)], nfull.value


# ---- plan ----

def cc_plan_create(tensors: Sequence[Tensor], R: int, chunk_elems: int = 0) -> Plan:
    return cc_plan_create_ex(tensors, R, chunk_elems, CC_GRAD_F16)


def cc_plan_create_ex(tensors: Sequence[Tensor], R: int, chunk_elems: int = 0, grad_dtype: int = CC_GRAD_F16) -> Plan:
    arr = (cc_tensor * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = _c_tensor(t)
    handle = C.c_void_p()
    _check(load().cc_plan_create_ex(arr, len(tensors), R, chunk_elems, grad_dtype, C.byref(handle)))
    return Plan(handle.value, list(tensors))


def cc_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def cc_plan_set_schedule(plan: Plan, schedule: int = CC_SCHEDULE_AUTO, workgroups: int = 0) -> None:
    _check(load().cc_plan_set_schedule(plan.handle, schedule, workgroups))


def cc_plan_schedule(plan: Plan):
    """(schedule the plan will use: CC_SCHEDULE_ORDERED or CC_SCHEDULE_PER_CHUNK, workgroups per launch)."""
    sched, wgs = C.c_int32(), C.c_int32()
    _check(load().cc_plan_schedule(plan.handle, C.byref(sched), C.byref(wgs)))
    return sched.value, wgs.value


def cc_plan_set_chunk_elems(plan: Plan, chunk_elems: int = 0) -> None:
    _check(load().cc_plan_set_chunk_elems(plan.handle, chunk_elems))


def cc_plan_layout(plan: Plan):
    """(chunk size in elements, threads per workgroup, CC_CACHE_STREAMING, CC_CACHE_RESIDENT or CC_CACHE_WRITE_THROUGH) the plan will use."""
    ce, blk, pol = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load().cc_plan_layout(plan.handle, C.byref(ce), C.byref(blk), C.byref(pol)))
    return ce.value, blk.value, pol.value


def cc_plan_set_cache_policy(plan: Plan, policy: int = CC_CACHE_AUTO) -> None:
    _check(load().cc_plan_set_cache_policy(plan.handle, policy))


def cc_plan_reserve_unfused(plan: Plan) -> None:
    _check(load().cc_plan_reserve_unfused(plan.handle))


def cc_plan_queue_state(plan: Plan, stream=None):
    """(ticket counter, finished-workgroup word) of the ordered schedule after waiting for the stream; both 0 between launches."""
    nxt, done = C.c_uint32(), C.c_uint64()
    _check(load().cc_plan_queue_state(plan.handle, C.byref(nxt), C.byref(done), _stream(stream)))
    return nxt.value, done.value


def cc_plan_autotune(plan: Plan, hp, flag, optimizer: int = 0, stream=None):
    """Times the candidate layouts and schedules on the plan's own buffers and keeps the fastest.  Returns (ms per step
    of what was kept, ms per step with one workgroup per chunk under the layout the plan had)."""
    c = _hp(hp)
    best, per_chunk = C.c_float(), C.c_float()
    _check(load().cc_plan_autotune(plan.handle, C.byref(c), optimizer, _ptr(flag), _stream(stream), C.byref(best), C.byref(per_chunk)))
    return best.value, per_chunk.value


def cc_plan_info(plan: Plan):
    numel, chunks, tb = C.c_uint64(), C.c_int64(), C.c_uint64()
    _check(load().cc_plan_info(plan.handle, C.byref(numel), C.byref(chunks), C.byref(tb)))
    return numel.value, chunks.value, tb.value


# ---- steps ----

def _step(name: str, plan: Plan, hp, flag, stream) -> None:
    c = _hp(hp)
    _check(getattr(load(), name)(plan.handle, C.byref(c), _ptr(flag), _stream(stream)))


def cc_fused_adam_step(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_fused_adam_step", plan, hp, flag, stream)


def cc_fused_adam_step_static(tensor: Tensor, R: int, hp, flag, stream=None) -> None:
    t, c = _c_tensor(tensor), _hp(hp)
    _check(load().cc_fused_adam_step_static(C.byref(t), R, C.byref(c), _ptr(flag), _stream(stream)))


def cc_fused_lamb_step(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_fused_lamb_step", plan, hp, flag, stream)


def cc_fused_lamb_phase1(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_fused_lamb_phase1", plan, hp, flag, stream)


def cc_fused_lamb_phase2(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_fused_lamb_phase2", plan, hp, flag, stream)


def cc_unfused_adam_step(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_unfused_adam_step", plan, hp, flag, stream)


def cc_unfused_adam_step_ex(plan: Plan, hp, flag, stream=None, sum_dtype: int = CC_GRAD_F32) -> None:
    c = _hp(hp)
    _check(load().cc_unfused_adam_step_ex(plan.handle, C.byref(c), _ptr(flag), _stream(stream), sum_dtype))


def cc_unfused_lamb_step(plan: Plan, hp, flag, stream=None) -> None:
    _step("cc_unfused_lamb_step", plan, hp, flag, stream)


def cc_lamb_norm_buffer(plan: Plan) -> int:
    p = C.c_void_p()
    _check(load().cc_lamb_norm_buffer(plan.handle, C.byref(p)))
    return p.value


def cc_lamb_norms_read(plan: Plan, T: int, stream=None):
    """Returns [(sum w^2, sum u^2)] per tensor after waiting for the stream."""
    buf = (C.c_double * max(2 * T, 2))()
    _check(load().cc_lamb_norms_read(plan.handle, buf, _stream(stream)))
    return [(buf[2 * i], buf[2 * i + 1]) for i in range(T)]


def _epilogue(partials, bias, residual, out, first: int, hidden: int, dropout_p: float, seed: int, numel=None) -> cc_epilogue:
    e = cc_epilogue()
    e.numel = residual.numel() if numel is None else numel
    e.first, e.hidden, e.R = first, hidden, len(partials)
    for r, x in enumerate(partials[:CC_MAX_R]):
        e.partial[r] = _ptr(x)
    e.bias, e.residual, e.out = _ptr(bias), _ptr(residual), _ptr(out)
    e.dropout_p, e.seed = dropout_p, seed
    return e


def cc_fused_epilogue(partials, bias, residual, out, first: int, hidden: int, dropout_p: float, seed: int, stream=None,
                      numel=None) -> None:
    e = _epilogue(partials, bias, residual, out, first, hidden, dropout_p, seed, numel)
    _check(load().cc_fused_epilogue(C.byref(e), _stream(stream)))


def cc_unfused_epilogue(partials, bias, residual, out, sum_scratch, first: int, hidden: int, dropout_p: float, seed: int,
                        stream=None, numel=None) -> None:
    e = _epilogue(partials, bias, residual, out, first, hidden, dropout_p, seed, numel)
    _check(load().cc_unfused_epilogue(C.byref(e), _ptr(sum_scratch), _stream(stream)))


def _c_tensor(t: Tensor) -> cc_tensor:
    c = cc_tensor()
    c.numel = t.numel
    c.w_in, c.m_in, c.v_in = _ptr(t.w_in), _ptr(t.m_in), _ptr(t.v_in)
    c.w_out, c.m_out, c.v_out = _ptr(t.w_out), _ptr(t.m_out), _ptr(t.v_out)
    c.w16_out = _ptr(t.w16_out)
    for r, g in enumerate(t.grad[:CC_MAX_R]):
        c.grad[r] = _ptr(g)
    c.weight_decay = t.weight_decay
    return c


def cc_pattern_probe(tensor: Tensor, R: int, what: int, cache_policy: int, sink, stream=None) -> None:
    c = _c_tensor(tensor)
    _check(load().cc_pattern_probe(C.byref(c), R, what, cache_policy, _ptr(sink), _stream(stream)))


def cc_copy_probe(dst, src, nbytes: int, stream=None) -> None:
    _check(load().cc_copy_probe(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def cc_device_info():
    """(compute units, memory clock kHz, memory bus bits, total bytes) of the current device."""
    cus, clk, bus, tot = C.c_int32(), C.c_int32(), C.c_int32(), C.c_uint64()
    _check(load().cc_device_info(C.byref(cus), C.byref(clk), C.byref(bus), C.byref(tot)))
    return cus.value, clk.value, bus.value, tot.value


def cc_last_error() -> str:
    return load().cc_last_error().decode()


def cc_version() -> int:
    return load().cc_version()
