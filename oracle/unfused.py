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
