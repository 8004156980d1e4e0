"""CPU fp64 oracle for jagged CROSS attention (queries and keys of a sample have their own lengths) -- test
infrastructure only.

The paper's feature-interaction use of attention is between a sample's feature values and its target items: two
jagged tensors with the same samples and different lengths.  With s_b = offsets_q[b], L_b = offsets_q[b + 1] - s_b
query rows and t_b = offsets_kv[b], M_b key rows of sample b, per head h:

  S_ij = q[s_b + i, h, :] . k[t_b + j, h, :] / sqrt(D)       (i < L_b, j < M_b)
  lse_i = log sum_j exp(S_ij),   P_ij = exp(S_ij - lse_i),   out[s_b + i, h, :] = sum_j P_ij v[t_b + j, h, :]
  backward, given dout:  delta_i = dout_i . out_i,  dV_j = sum_i P_ij dout_i,  dS_ij = P_ij (dout_i . v_j - delta_i),
                         dq_i = sum_j dS_ij k_j / sqrt(D),  dk_j = sum_i dS_ij q_i / sqrt(D)

A sample without keys (M_b = 0) has an empty softmax: out = 0, lse = -inf and no gradient flows.  With equal offsets
this is the self-attention of oracle/jfa_oracle.c (a different program; the pins compare the two).
Plain numpy, one (sample, head) at a time, full score matrix in memory.
"""
from __future__ import annotations

import numpy as np


def _prep(q, k, v, offsets_q, offsets_kv):
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    oq, ok = np.asarray(offsets_q, dtype=np.int64), np.asarray(offsets_kv, dtype=np.int64)
    assert len(oq) == len(ok) and q.shape[1:] == k.shape[1:] == v.shape[1:] and k.shape == v.shape
    return q, k, v, oq, ok


def _probs(qb, kb):
    """P [L, M] and lse [L] of one (sample, head); M >= 1."""
    s = (qb @ kb.T) / np.sqrt(qb.shape[1])
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def forward(q, k, v, offsets_q, offsets_kv):
    q, k, v, oq, ok = _prep(q, k, v, offsets_q, offsets_kv)
    nq, H, D = q.shape
    out = np.zeros((nq, H, D))
    lse = np.full((H, nq), -np.inf)
    for b in range(len(oq) - 1):
        s, e, t, u = int(oq[b]), int(oq[b + 1]), int(ok[b]), int(ok[b + 1])
        if e == s or u == t:
            continue
        for h in range(H):
            p, lse[h, s:e] = _probs(q[s:e, h], k[t:u, h])
            out[s:e, h] = p @ v[t:u, h]
    return out, lse


def backward(q, k, v, dout, offsets_q, offsets_kv):
    q, k, v, oq, ok = _prep(q, k, v, offsets_q, offsets_kv)
    dout = np.asarray(dout, dtype=np.float64)
    nq, H, D = q.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    delta = np.zeros((H, nq))
    for b in range(len(oq) - 1):
        s, e, t, u = int(oq[b]), int(oq[b + 1]), int(ok[b]), int(ok[b + 1])
        if e == s or u == t:
            continue
        for h in range(H):
            p, _ = _probs(q[s:e, h], k[t:u, h])
            o = p @ v[t:u, h]
            dl = (dout[s:e, h] * o).sum(axis=1)
            delta[h, s:e] = dl
            dv[t:u, h] = p.T @ dout[s:e, h]
            ds = p * (dout[s:e, h] @ v[t:u, h].T - dl[:, None])
            dq[s:e, h] = ds @ k[t:u, h] / np.sqrt(D)
            dk[t:u, h] = ds.T @ q[s:e, h] / np.sqrt(D)
    return dq, dk, dv, delta
