"""Shared helpers of the test suite: array builders and the comparison rules of the parity bar."""
from __future__ import annotations

import numpy as np

import oracle

REL_TOL = 2e-6          # fp32 master weights, m and v against the fp64 oracle


def f32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def half_bits(x):
    """fp16 bit patterns (uint16) of real values, rounded by numpy (round to nearest even)."""
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16))


def bits_to_f64(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def make_tensor(w, grads_bits, m=None, v=None, wd=0.0):
    w = f32(w)
    m = np.zeros_like(w) if m is None else f32(m)
    v = np.zeros_like(w) if v is None else f32(v)
    # uint16 arrays are fp16 bit patterns; float32 arrays are fp32 gradient slices
    grads = [np.ascontiguousarray(g) if getattr(g, "dtype", None) == np.float32 else np.ascontiguousarray(np.asarray(g, dtype=np.uint16))
             for g in grads_bits]
    return oracle.OracleTensor(w=w, m=m, v=v, grads=grads, weight_decay=wd)


def fl(x):
    """Round float64 values to fp32 (nearest even) and return them as float64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def ulp_f32(a, b):
    """Distance in fp32 units in the last place between two float32 arrays (order-preserving integer map)."""
    def key(x):
        i = np.asarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, np.int64(-(2 ** 31)) - i, i)
    return np.abs(key(a) - key(b))


def half_ulp_distance(a_bits, b_bits):
    """Distance between fp16 bit patterns on the ordered fp16 line; two non-finite values count as equal."""
    a = np.asarray(a_bits, dtype=np.uint16).astype(np.int64)
    b = np.asarray(b_bits, dtype=np.uint16).astype(np.int64)

    def key(x):
        mag = x & 0x7FFF
        return np.where((x & 0x8000) != 0, -mag, mag)
    d = np.abs(key(a) - key(b))
    both_nonfinite = ((a & 0x7C00) == 0x7C00) & ((b & 0x7C00) == 0x7C00)
    return np.where(both_nonfinite, 0, d)


def state_error(x, y):
    """Violation ratio of the fp32 parity rule: |x-y| / (REL_TOL * max(|y|, rms(y))), elementwise max.

    y is the oracle's tensor.  The rms floor covers the few elements where beta*m and (1-beta)*g cancel,
    so that the bound stays relative to the size of the terms that were actually rounded.
    Returns (worst ratio, worst pure relative error, count of elements above REL_TOL in pure relative terms).
    """
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    if x.size == 0:
        return 0.0, 0.0, 0
    if not np.array_equal(np.isfinite(x), np.isfinite(y)):
        return np.inf, np.inf, int(np.sum(np.isfinite(x) != np.isfinite(y)))
    fin = np.isfinite(y)
    x, y = x[fin], y[fin]
    if x.size == 0:
        return 0.0, 0.0, 0
    rms = float(np.sqrt(np.mean(y * y)))
    diff = np.abs(x - y)
    floor = np.maximum(np.abs(y), rms)
    ratio = diff / (REL_TOL * np.where(floor > 0, floor, 1.0))
    ratio = np.where((floor == 0) & (diff == 0), 0.0, ratio)
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(y != 0, diff / np.abs(y), np.where(diff == 0, 0.0, np.inf))
    return float(ratio.max()), float(rel.max()), int(np.sum(rel > REL_TOL))
