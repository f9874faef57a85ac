"""CPU oracle for HAG aggregation -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``hag_oracle.c`` (plain C, fp64 accumulation).
Nothing here is shared with, imports, or is imported by the HIP library: only
``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg use it.

Each function names the passage of the paper it follows; the arithmetic itself
is in the C file, which states the conventions taken where the paper is silent.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hag_oracle.c")
_LIB = os.path.join(_HERE, "libhag_oracle.so")

OP_SUM, OP_MEAN, OP_MAX, OP_GCN = 0, 1, 2, 3
_OPS = {"sum": OP_SUM, "mean": OP_MEAN, "max": OP_MAX, "gcn": OP_GCN}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (-O2, OpenMP on independent loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_search.restype = ctypes.c_int64
        _lib.oracle_cover_check.restype = ctypes.c_int64
        _lib.oracle_redundancy.restype = ctypes.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(x):
    return ctypes.c_int64(int(x))


def _csr(rowptr, col):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    return rowptr, col


def naive_forward(rowptr, col, x, op="sum"):
    """Algorithm 1, Aggregate line, with the set aggregates of Table 1 (+ mean); op "gcn" is
    Table 1's GCN row up to the weight matrix: (sum over N(v) of h_u + h_v) / (|N(v)| + 1).

    fp32 ``x`` -> (y float64, s_abs float64, argmax int32 or None);
    int32 ``x`` -> (y int32, None, argmax or None)."""
    lib = _load()
    rowptr, col = _csr(rowptr, col)
    n = rowptr.size - 1
    x = np.ascontiguousarray(x)
    d = x.shape[1]
    o = _OPS[op]
    am = np.full((n, d), -1, dtype=np.int32) if o == OP_MAX else None
    if x.dtype == np.float32:
        y = np.zeros((n, d), dtype=np.float64)
        s = np.zeros((n, d), dtype=np.float64)
        lib.oracle_naive_forward_f32(_i64(n), _p(rowptr), _p(col), _i64(d), o, _p(x), _p(y), _p(s), _p(am))
        return y, s, am
    if x.dtype == np.int32:
        if o in (OP_MEAN, OP_GCN):
            raise ValueError("mean / gcn are not defined for int32")
        y = np.zeros((n, d), dtype=np.int32)
        lib.oracle_naive_forward_i32(_i64(n), _p(rowptr), _p(col), _i64(d), o, _p(x), _p(y), _p(am))
        return y, None, am
    raise TypeError(x.dtype)


def naive_backward(rowptr, col, gy, op="sum", argmax=None):
    """Vector-Jacobian product of :func:`naive_forward` (equivalence, Section 3.2,
    requires the HAG path to return exactly this gradient).

    fp32 -> (gx float64, s_abs float64); int32 -> (gx int32, None)."""
    lib = _load()
    rowptr, col = _csr(rowptr, col)
    n = rowptr.size - 1
    gy = np.ascontiguousarray(gy)
    d = gy.shape[1]
    o = _OPS[op]
    if o == OP_MAX:
        argmax = np.ascontiguousarray(argmax, dtype=np.int32)
    if gy.dtype == np.float32:
        gx = np.zeros((n, d), dtype=np.float64)
        s = np.zeros((n, d), dtype=np.float64)
        lib.oracle_naive_backward_f32(_i64(n), _p(rowptr), _p(col), _i64(d), o, _p(gy), _p(argmax), _p(gx), _p(s))
        return gx, s
    if gy.dtype == np.int32:
        gx = np.zeros((n, d), dtype=np.int32)
        lib.oracle_naive_backward_i32(_i64(n), _p(rowptr), _p(col), _i64(d), o, _p(gy), _p(argmax), _p(gx))
        return gx, None
    raise TypeError(gy.dtype)


class Hag:
    """A HAG in creation order (unified ids: originals 0..n-1, aggregation nodes n..n+a-1).

    ``left/right[i]`` are the two in-neighbours of aggregation node ``n+i``;
    ``hrowptr/hcol`` hold the HAG in-neighbours of every original node."""

    def __init__(self, n, left, right, hrowptr, hcol, red=None):
        self.n = int(n)
        self.left = np.ascontiguousarray(left, dtype=np.int32)
        self.right = np.ascontiguousarray(right, dtype=np.int32)
        self.a = int(self.left.size)
        self.hrowptr = np.ascontiguousarray(hrowptr, dtype=np.int64)
        self.hcol = np.ascontiguousarray(hcol, dtype=np.int32)
        self.red = None if red is None else np.ascontiguousarray(red, dtype=np.int32)

    # Section 4.1: computing a node with k in-neighbours takes k-1 binary aggregations
    def aggregations(self) -> int:
        k = np.diff(self.hrowptr)
        return int(np.maximum(k - 1, 0).sum()) + self.a  # each aggregation node: 2 - 1

    def edges(self) -> int:
        return int(self.hcol.size) + 2 * self.a


def hag_forward(h: Hag, deg, x, op="sum"):
    """Algorithm 2: copy loop, aggregation-node loop (creation order), final loop."""
    lib = _load()
    x = np.ascontiguousarray(x)
    d = x.shape[1]
    o = _OPS[op]
    deg = np.ascontiguousarray(deg, dtype=np.int64)
    am = np.full((h.n, d), -1, dtype=np.int32) if o == OP_MAX else None
    if x.dtype == np.float32:
        y = np.zeros((h.n, d), dtype=np.float64)
        lib.oracle_hag_forward_f32(_i64(h.n), _i64(h.a), _p(h.left), _p(h.right), _p(h.hrowptr), _p(h.hcol),
                                   _p(deg), _i64(d), o, _p(x), _p(y), _p(am))
        return y, am
    if x.dtype == np.int32:
        y = np.zeros((h.n, d), dtype=np.int32)
        lib.oracle_hag_forward_i32(_i64(h.n), _i64(h.a), _p(h.left), _p(h.right), _p(h.hrowptr), _p(h.hcol),
                                   _i64(d), o, _p(x), _p(y), _p(am))
        return y, am
    raise TypeError(x.dtype)


def hag_backward(h: Hag, deg, gy, op="sum"):
    """Reverse of Algorithm 2 for sum / mean (max back-propagates through argmax only)."""
    lib = _load()
    gy = np.ascontiguousarray(gy)
    d = gy.shape[1]
    o = _OPS[op]
    if o == OP_MAX:
        raise ValueError("max backward needs no HAG: use naive_backward with argmax")
    deg = np.ascontiguousarray(deg, dtype=np.int64)
    if gy.dtype == np.float32:
        gx = np.zeros((h.n, d), dtype=np.float64)
        lib.oracle_hag_backward_f32(_i64(h.n), _i64(h.a), _p(h.left), _p(h.right), _p(h.hrowptr), _p(h.hcol),
                                    _p(deg), _i64(d), o, _p(gy), _p(gx))
        return gx
    if gy.dtype == np.int32:
        gx = np.zeros((h.n, d), dtype=np.int32)
        lib.oracle_hag_backward_i32(_i64(h.n), _i64(h.a), _p(h.left), _p(h.right), _p(h.hrowptr), _p(h.hcol),
                                    _i64(d), _p(gy), _p(gx))
        return gx
    raise TypeError(gy.dtype)


def cover_check(rowptr, col, h: Hag) -> int:
    """Equation 1 expanded as a multiset, compared with N(v) for every v (Theorem 2).

    0 = equivalent; 1+v = first node whose cover differs; -1 = malformed HAG."""
    lib = _load()
    rowptr, col = _csr(rowptr, col)
    return int(lib.oracle_cover_check(_i64(h.n), _p(rowptr), _p(col), _i64(h.a), _p(h.left), _p(h.right),
                                      _p(h.hrowptr), _p(h.hcol)))


def search(rowptr, col, capacity) -> Hag:
    """Algorithm 3 (set Aggregate) by brute force: all pairs recounted every iteration.

    Memory is (n+capacity)^2 counters -- small graphs only."""
    lib = _load()
    rowptr, col = _csr(rowptr, col)
    n = rowptr.size - 1
    capacity = int(capacity)
    if (n + capacity) ** 2 > 4 * 10**8:
        raise ValueError("oracle search is brute force: graph too large")
    left = np.zeros(max(capacity, 1), dtype=np.int32)
    right = np.zeros(max(capacity, 1), dtype=np.int32)
    red = np.zeros(max(capacity, 1), dtype=np.int32)
    hrowptr = np.zeros(n + 1, dtype=np.int64)
    hcol = np.zeros(max(col.size, 1), dtype=np.int32)
    a = int(lib.oracle_search(_i64(n), _p(rowptr), _p(col), _i64(capacity), _p(left), _p(right), _p(red),
                              _p(hrowptr), _p(hcol)))
    return Hag(n, left[:a], right[:a], hrowptr, hcol[: hrowptr[n]], red[:a])


def redundancy(n, hrowptr, hcol, v1, v2) -> int:
    """Redundancy(v1, v2) of Algorithm 3 for a set Aggregate."""
    lib = _load()
    hrowptr, hcol = _csr(hrowptr, hcol)
    return int(lib.oracle_redundancy(_i64(n), _p(hrowptr), _p(hcol), ctypes.c_int32(v1), ctypes.c_int32(v2)))
