"""CPU fp64 oracle for jagged attention -- test infrastructure only (tests, smoke, bench cpu_baseline).

Thin ctypes wrapper around ``jfa_oracle.c`` (compiled with gcc by ``oracle.build()``).
It never imports the HIP package and the HIP package never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jfa_oracle.c")
_LIB = os.path.join(_HERE, "libjfa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, -O2, no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB + ".tmp", _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.jfa_oracle_forward.restype = ctypes.c_int
        lib.jfa_oracle_forward.argtypes = [f32p, f32p, f32p, i64p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                           i64p, i32p, ctypes.c_int64, f64p, f64p]
        lib.jfa_oracle_backward.restype = ctypes.c_int
        lib.jfa_oracle_backward.argtypes = [f32p, f32p, f32p, f32p, i64p, ctypes.c_int64, ctypes.c_int,
                                            ctypes.c_int, i64p, i32p, ctypes.c_int64, f64p, f64p, f64p, f64p]
        lib.jfa_oracle_probs.restype = None
        lib.jfa_oracle_probs.argtypes = [f32p, f32p, f32p, i64p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int64, ctypes.c_int, f64p]
        _lib = lib
    return _lib


def _f32(x):
    a = np.ascontiguousarray(x, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _pairs(pairs):
    if pairs is None:
        return None, None, 0, None
    pb = np.ascontiguousarray([p[0] for p in pairs], dtype=np.int64)
    ph = np.ascontiguousarray([p[1] for p in pairs], dtype=np.int32)
    return (pb.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ph.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
            len(pairs), (pb, ph))


def _check(q, k, v, offsets):
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    assert q.ndim == 3 and q.shape == k.shape == v.shape, "q, k, v must be [sum_B, H, D]"
    assert offsets.ndim == 1 and offsets[0] == 0 and np.all(np.diff(offsets) >= 0), "bad offsets"
    assert offsets[-1] <= q.shape[0], "offsets[B] exceeds the number of rows"
    return offsets


def forward(q, k, v, offsets, pairs: Optional[Sequence[Tuple[int, int]]] = None, return_threads: bool = False):
    """out [sum_B, H, D] fp64 and lse [H, sum_B] fp64.

    ``pairs`` restricts the work to the listed (sample, head) pairs; every other row is NaN.
    Rows of q/k/v beyond ``offsets[-1]`` are never read.
    """
    lib = _load()
    offsets = _check(q, k, v, offsets)
    B = len(offsets) - 1
    sum_B = int(offsets[-1])
    _, H, D = q.shape
    qa, qp = _f32(q); ka, kp = _f32(k); va, vp = _f32(v)
    out = np.full((sum_B, H, D), np.nan, dtype=np.float64)
    lse = np.full((H, sum_B), np.nan, dtype=np.float64)
    pb, ph, n, keep = _pairs(pairs)
    threads = lib.jfa_oracle_forward(qp, kp, vp, offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), B, H, D,
                                     pb, ph, n, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                     lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    del keep
    return (out, lse, threads) if return_threads else (out, lse)


def backward(q, k, v, dout, offsets, pairs: Optional[Sequence[Tuple[int, int]]] = None):
    """dq, dk, dv [sum_B, H, D] fp64 and delta [H, sum_B] fp64 (rows of unlisted pairs are NaN)."""
    lib = _load()
    offsets = _check(q, k, v, offsets)
    assert dout.shape == q.shape
    B = len(offsets) - 1
    sum_B = int(offsets[-1])
    _, H, D = q.shape
    qa, qp = _f32(q); ka, kp = _f32(k); va, vp = _f32(v); da, dp = _f32(dout)
    f64p = ctypes.POINTER(ctypes.c_double)
    dq = np.full((sum_B, H, D), np.nan, dtype=np.float64)
    dk = np.full((sum_B, H, D), np.nan, dtype=np.float64)
    dv = np.full((sum_B, H, D), np.nan, dtype=np.float64)
    delta = np.full((H, sum_B), np.nan, dtype=np.float64)
    pb, ph, n, keep = _pairs(pairs)
    lib.jfa_oracle_backward(qp, kp, vp, dp, offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), B, H, D,
                            pb, ph, n, dq.ctypes.data_as(f64p), dk.ctypes.data_as(f64p), dv.ctypes.data_as(f64p),
                            delta.ctypes.data_as(f64p))
    del keep
    return dq, dk, dv, delta


def probs(q, k, v, offsets, b: int, h: int):
    """The L_b x L_b softmax matrix of one (sample, head) in fp64 (tiny cases)."""
    lib = _load()
    offsets = _check(q, k, v, offsets)
    B = len(offsets) - 1
    _, H, D = q.shape
    L = int(offsets[b + 1] - offsets[b])
    qa, qp = _f32(q); ka, kp = _f32(k); va, vp = _f32(v)
    P = np.zeros((L, L), dtype=np.float64)
    lib.jfa_oracle_probs(qp, kp, vp, offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), B, H, D, b, h,
                         P.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return P
