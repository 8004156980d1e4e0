"""Pins for oracle/causal.py (causal jagged self attention).

  Z1  torch fp64 scaled_dot_product_attention(is_causal=True) per sample, gradients by autograd
  Z2  causality: the first n rows of a sample's output (and lse) equal the output of the sample cut to n rows
      computed by the NON-causal C oracle's last row trick -- row i of causal attention is the last row of
      non-causal attention over rows 0..i (another program)
  Z3  closed forms: row 0 returns v_0 with lse = S_00; the last key only receives gradient from the last query
      (dv of the last row = P_last,last * dout_last)
  Z4  samples of length 0 and 1
"""
import numpy as np
import torch

from oracle import causal


def _data(L, H, D, seed=0):
    rng = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(L)])
    mk = lambda: rng.standard_normal((off[-1], H, D))
    return mk(), mk(), mk(), mk(), off


def test_z1_torch_sdpa_causal():
    L = [6, 1, 0, 11, 3]
    q, k, v, do, off = _data(L, 2, 4, seed=1)
    qt, kt, vt = (torch.from_numpy(a).requires_grad_(True) for a in (q, k, v))
    outs = []
    for b in range(len(L)):
        if L[b]:
            a = [x[off[b]:off[b + 1]].transpose(0, 1) for x in (qt, kt, vt)]
            outs.append(torch.nn.functional.scaled_dot_product_attention(*a, is_causal=True).transpose(0, 1))
    out_t = torch.cat(outs)
    (out_t * torch.from_numpy(do)).sum().backward()
    out, lse = causal.forward(q, k, v, off)
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-12, atol=1e-13)
    dq, dk, dv, delta = causal.backward(q, k, v, do, off)
    np.testing.assert_allclose(dq, qt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dk, kt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dv, vt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(delta, (do * out).sum(axis=2).T, rtol=1e-12, atol=1e-13)


def test_z2_each_row_is_the_last_row_of_a_prefix(oracle):
    L = [9, 4]
    q, k, v, _, off = _data(L, 2, 8, seed=2)
    q, k, v = (a.astype(np.float32) for a in (q, k, v))
    out, lse = causal.forward(q, k, v, off)
    for b in range(2):
        s = off[b]
        for i in range(L[b]):
            o_c, l_c = oracle.forward(q[s:s + i + 1], k[s:s + i + 1], v[s:s + i + 1], np.array([0, i + 1]))
            np.testing.assert_allclose(out[s + i], o_c[i], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[:, s + i], l_c[:, i], rtol=1e-12, atol=1e-13)


def test_z3_closed_forms():
    q, k, v, do, off = _data([5], 1, 4, seed=3)
    out, lse = causal.forward(q, k, v, off)
    np.testing.assert_allclose(out[0], v[0], rtol=1e-15)
    np.testing.assert_allclose(lse[0, 0], q[0, 0] @ k[0, 0] / 2.0, rtol=1e-14)
    _, _, dv, _ = causal.backward(q, k, v, do, off)
    s_last = q[4, 0] @ k[:, 0].T / 2.0
    p_last = np.exp(s_last[4] - np.log(np.exp(s_last).sum()))
    np.testing.assert_allclose(dv[4, 0], p_last * do[4, 0], rtol=1e-13)


def test_z4_lengths_zero_and_one():
    q, k, v, do, off = _data([0, 1, 0], 2, 4, seed=4)
    out, lse = causal.forward(q, k, v, off)
    np.testing.assert_allclose(out, v, rtol=1e-15)
    dq, dk, dv, _ = causal.backward(q, k, v, do, off)
    np.testing.assert_allclose(dv, do, rtol=1e-15)
    np.testing.assert_allclose(dq, 0.0, atol=1e-15)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)
