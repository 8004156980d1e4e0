"""CPU fp64 oracle for the UNFUSED jagged attention (paper Table 1's three attention rows) -- test infrastructure only.

The paper's "jagged attention" baseline runs attention as three separate jagged operators and writes the score
array to memory (Table 1: a jagged x jagged product with a jagged square output, a softmax over that output,
and a product of that output with a jagged tensor; Section 3 compares the fused kernel with it).  Each
function below is the plain definition of one of them, per sample and head, in fp64 numpy:

  scores(q, k, offsets)        S[h, sq[b] + i * L_b + j] = sum_d q[s_b + i, h, d] k[s_b + j, h, d] / sqrt(D)
  softmax_rows(S, offsets)     P[h, sq[b] + i * L_b + j] = exp(S_ij - max_j S_ij) / sum_j exp(S_ij - max_j S_ij)
  apply(P, v, offsets)         out[s_b + i, h, d] = sum_j P[h, sq[b] + i * L_b + j] v[s_b + j, h, d]

with s_b = offsets[b], L_b = offsets[b + 1] - offsets[b] and sq = [0, cumsum(L_b^2)] (square_offsets).
Their composition is the attention forward of oracle/jfa_oracle.c (a different program in a different
language: tests/test_oracle_pins.py checks that they agree).

The paper builds forward and backward for its jagged operators (Section 2.2).  The gradients of the three are
products of the same kinds plus the softmax's own backward:

  product(a, b, offsets, scale)            X[h, sq[b] + i * L_b + j] = scale * a[s_b + i, h, :] . b[s_b + j, h, :]
                                           (scores is product(q, k, 1 / sqrt(D)); dP = product(dout, v, 1))
  softmax_rows_backward(P, dP, offsets, scale)   dS_ij = scale * P_ij (dP_ij - sum_j' P_ij' dP_ij')
  apply_transposed(X, x, offsets)          out[s_b + j, h, :] = sum_i X[h, sq[b] + i * L_b + j] x[s_b + i, h, :]
                                           (dV = apply_transposed(P, dout); dK = apply_transposed(dS, q))
  and dQ = apply(dS, k), with dS scaled by 1 / sqrt(D) in softmax_rows_backward.
"""
from __future__ import annotations

import numpy as np


def square_offsets(offsets) -> np.ndarray:
    L = np.diff(np.asarray(offsets, dtype=np.int64))
    return np.concatenate([[0], np.cumsum(L * L)]).astype(np.int64)


def scores(q, k, offsets) -> np.ndarray:
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    _, H, D = q.shape
    sq = square_offsets(offsets)
    S = np.zeros((H, int(sq[-1])), dtype=np.float64)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        L = e - s
        for h in range(H):
            S[h, sq[b]:sq[b + 1]] = ((q[s:e, h, :] @ k[s:e, h, :].T) / np.sqrt(D)).reshape(L * L)
    return S


def product(a, b, offsets, scale: float) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    H = a.shape[1]
    sq = square_offsets(offsets)
    X = np.zeros((H, int(sq[-1])), dtype=np.float64)
    for s_idx in range(len(offsets) - 1):
        s, e = int(offsets[s_idx]), int(offsets[s_idx + 1])
        for h in range(H):
            X[h, sq[s_idx]:sq[s_idx + 1]] = (scale * (a[s:e, h, :] @ b[s:e, h, :].T)).reshape((e - s) ** 2)
    return X


def softmax_rows_backward(P, dP, offsets, scale: float = 1.0) -> np.ndarray:
    P = np.asarray(P, dtype=np.float64)
    dP = np.asarray(dP, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    sq = square_offsets(offsets)
    dS = np.zeros_like(P)
    for b in range(len(offsets) - 1):
        L = int(offsets[b + 1] - offsets[b])
        if L == 0:
            continue
        p = P[:, sq[b]:sq[b + 1]].reshape(P.shape[0], L, L)
        g = dP[:, sq[b]:sq[b + 1]].reshape(P.shape[0], L, L)
        dS[:, sq[b]:sq[b + 1]] = (scale * p * (g - (p * g).sum(axis=2, keepdims=True))).reshape(P.shape[0], L * L)
    return dS


def apply_transposed(X, x, offsets) -> np.ndarray:
    X = np.asarray(X, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    n, H, D = x.shape
    sq = square_offsets(offsets)
    out = np.zeros((n, H, D), dtype=np.float64)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        L = e - s
        for h in range(H):
            out[s:e, h, :] = X[h, sq[b]:sq[b + 1]].reshape(L, L).T @ x[s:e, h, :]
    return out


def softmax_rows(S, offsets) -> np.ndarray:
    S = np.asarray(S, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    sq = square_offsets(offsets)
    P = np.zeros_like(S)
    for b in range(len(offsets) - 1):
        L = int(offsets[b + 1] - offsets[b])
        if L == 0:
            continue
        blk = S[:, sq[b]:sq[b + 1]].reshape(S.shape[0], L, L)
        blk = blk - blk.max(axis=2, keepdims=True)
        ex = np.exp(blk)
        P[:, sq[b]:sq[b + 1]] = (ex / ex.sum(axis=2, keepdims=True)).reshape(S.shape[0], L * L)
    return P


def apply(P, v, offsets) -> np.ndarray:
    P = np.asarray(P, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    offsets = np.asarray(offsets, dtype=np.int64)
    n, H, D = v.shape
    sq = square_offsets(offsets)
    out = np.zeros((n, H, D), dtype=np.float64)
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        L = e - s
        for h in range(H):
            out[s:e, h, :] = P[h, sq[b]:sq[b + 1]].reshape(L, L) @ v[s:e, h, :]
    return out
