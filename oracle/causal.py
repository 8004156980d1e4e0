"""CPU fp64 oracle for CAUSAL jagged self attention -- test infrastructure only.

Row i of a sample attends to rows j <= i of the same sample (the order of a sample's rows is the order of the
sequence).  With s_b = offsets[b] and L_b rows, per head h and i, j < L_b:

  S_ij = q[s_b + i, h, :] . k[s_b + j, h, :] / sqrt(D)  for j <= i,   excluded from the softmax for j > i
  lse_i = log sum_{j <= i} exp(S_ij),   P_ij = exp(S_ij - lse_i),   out[s_b + i] = sum_{j <= i} P_ij v[s_b + j]
  backward:  delta_i = dout_i . out_i,  dV_j = sum_{i >= j} P_ij dout_i,  dS_ij = P_ij (dout_i . v_j - delta_i),
             dq_i = sum_{j <= i} dS_ij k_j / sqrt(D),   dk_j = sum_{i >= j} dS_ij q_i / sqrt(D)

Plain numpy, one (sample, head) at a time, the full masked score matrix in memory.
"""
from __future__ import annotations

import numpy as np


def _probs(qb, kb):
    L = qb.shape[0]
    s = (qb @ kb.T) / np.sqrt(qb.shape[1])
    s = np.where(np.arange(L)[None, :] <= np.arange(L)[:, None], s, -np.inf)
    m = s.max(axis=1, keepdims=True)          # the diagonal is never masked: finite
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def forward(q, k, v, offsets):
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    offsets = np.asarray(offsets, dtype=np.int64)
    n, H, D = q.shape
    out, lse = np.zeros((n, H, D)), np.zeros((H, n))
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        for h in range(H):
            if e > s:
                p, lse[h, s:e] = _probs(q[s:e, h], k[s:e, h])
                out[s:e, h] = p @ v[s:e, h]
    return out, lse


def backward(q, k, v, dout, offsets):
    q, k, v, dout = (np.asarray(a, dtype=np.float64) for a in (q, k, v, dout))
    offsets = np.asarray(offsets, dtype=np.int64)
    n, H, D = q.shape
    dq, dk, dv, delta = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v), np.zeros((H, n))
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        for h in range(H):
            if e == s:
                continue
            p, _ = _probs(q[s:e, h], k[s:e, h])
            dl = (dout[s:e, h] * (p @ v[s:e, h])).sum(axis=1)
            delta[h, s:e] = dl
            dv[s:e, h] = p.T @ dout[s:e, h]
            ds = p * (dout[s:e, h] @ v[s:e, h].T - dl[:, None])
            dq[s:e, h] = ds @ k[s:e, h] / np.sqrt(D)
            dk[s:e, h] = ds.T @ q[s:e, h] / np.sqrt(D)
    return dq, dk, dv, delta
