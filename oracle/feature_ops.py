"""CPU fp64 oracle for the jagged feature operators of the paper's Table 1 -- test infrastructure only.

x is a jagged tensor [sum_B, D] with offsets [B + 1]; s_b = offsets[b], L_b = offsets[b + 1] - s_b.

  jagged_dense_bmm(x, w, offsets)     x [sum_B, D], w [B, D, T]     ->  out[s_b + i, t] = sum_d x[s_b + i, d] w[b, d, t]
  jagged_jagged_bmm(x, y, offsets)    x [sum_B, D], y [sum_B, T]    ->  out[b, d, t] = sum_{i < L_b} x[s_b + i, d] y[s_b + i, t]
  jagged_softmax(x, offsets)          x [sum_B, D]                  ->  y[s_b + i, d] = exp(x[s_b + i, d]) / sum_{j < L_b} exp(x[s_b + j, d])
  jagged_softmax_backward(y, dy, offsets)                           ->  dx[s_b + i, d] = y (dy - sum_{j < L_b} dy[s_b + j, d] y[s_b + j, d])

(Table 1 gives the shapes; the softmax of a jagged tensor runs along each sample's jagged dimension, one column at
a time.)  jagged_jagged_bmm is the gradient of jagged_dense_bmm with respect to w (with y = the output's gradient),
and jagged_dense_bmm with w transposed is its gradient with respect to x.  Each function is the plain definition,
one sample at a time; an empty sample gives a zero [D, T] block and no rows.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def jagged_dense_bmm(x, w, offsets) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    offsets = np.asarray(offsets, dtype=np.int64)
    out = np.zeros((x.shape[0], w.shape[2]), dtype=np.float64)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        out[s:e] = x[s:e] @ w[b]
    return out


def jagged_jagged_bmm(x, y, offsets) -> np.ndarray:
    x, y = _f64(x), _f64(y)
    offsets = np.asarray(offsets, dtype=np.int64)
    B = len(offsets) - 1
    out = np.zeros((B, x.shape[1], y.shape[1]), dtype=np.float64)
    for b in range(B):
        s, e = int(offsets[b]), int(offsets[b + 1])
        out[b] = x[s:e].T @ y[s:e]
    return out


def jagged_softmax(x, offsets) -> np.ndarray:
    x = _f64(x)
    offsets = np.asarray(offsets, dtype=np.int64)
    y = np.zeros_like(x)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        if e == s:
            continue
        z = np.exp(x[s:e] - x[s:e].max(axis=0, keepdims=True))
        y[s:e] = z / z.sum(axis=0, keepdims=True)
    return y


def jagged_softmax_backward(y, dy, offsets) -> np.ndarray:
    y, dy = _f64(y), _f64(dy)
    offsets = np.asarray(offsets, dtype=np.int64)
    dx = np.zeros_like(y)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        dx[s:e] = y[s:e] * (dy[s:e] - (dy[s:e] * y[s:e]).sum(axis=0, keepdims=True))
    return dx
