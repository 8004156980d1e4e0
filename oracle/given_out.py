"""CPU fp64 oracle for the backward pass AS THE INTERFACE DEFINES IT -- test infrastructure only.

jfa_backward receives the forward's output tensor and forms delta from it (paper Section 2.2 gives no equations; the
standard backward of Section 2.1's attention uses delta_i = dout_i . out_i).  With the `out` it is handed (a bf16
tensor on the GPU path, i.e. the exact output rounded once), per sample b (rows s_b .. s_b + L_b - 1), head h:

  S_ij = q_i . k_j / sqrt(D)  (j <= i only if causal),   P = row softmax of S       (from q, k: exact)
  delta_i = dout_i . out_i                                                           (from the GIVEN out)
  dV_j = sum_i P_ij dout_i,   dS_ij = P_ij (dout_i . v_j - delta_i),
  dq_i = sum_j dS_ij k_j / sqrt(D),   dk_j = sum_i dS_ij q_i / sqrt(D)

Given the exact fp64 output this is the plain backward of jfa_oracle.c / oracle.causal (the pin); given a rounded
output it shows how much of a gradient's error is inherited from that rounding rather than made by a kernel.
Plain numpy, one (sample, head) at a time, the full score matrix in memory.
"""
from __future__ import annotations

import numpy as np


def backward(q, k, v, out, dout, offsets, causal: bool = False):
    q, k, v, out, dout = (np.asarray(a, dtype=np.float64) for a in (q, k, v, out, dout))
    offsets = np.asarray(offsets, dtype=np.int64)
    n, H, D = q.shape
    dq, dk, dv, delta = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v), np.zeros((H, n))
    for b in range(len(offsets) - 1):
        s, e = int(offsets[b]), int(offsets[b + 1])
        L = e - s
        for h in range(H):
            if L == 0:
                continue
            S = (q[s:e, h] @ k[s:e, h].T) / np.sqrt(D)
            if causal:
                S = np.where(np.arange(L)[None, :] <= np.arange(L)[:, None], S, -np.inf)
            E = np.exp(S - S.max(axis=1, keepdims=True))
            P = E / E.sum(axis=1, keepdims=True)
            dl = (dout[s:e, h] * out[s:e, h]).sum(axis=1)
            delta[h, s:e] = dl
            dv[s:e, h] = P.T @ dout[s:e, h]
            dS = P * (dout[s:e, h] @ v[s:e, h].T - dl[:, None])
            dq[s:e, h] = dS @ k[s:e, h] / np.sqrt(D)
            dk[s:e, h] = dS.T @ q[s:e, h] / np.sqrt(D)
    return dq, dk, dv, delta
