"""Pins for oracle/cross.py (jagged cross attention: separate query and key lengths per sample).

  X1  with equal offsets it is the self-attention of the C oracle (another program in another language), forward
      and backward
  X2  torch fp64 scaled_dot_product_attention per sample with L_b != M_b, gradients by autograd
  X3  closed forms: a single key returns its value row and lse = the score; equal keys give the mean of the values and
      lse = score + log M; permuting a sample's keys (and values) changes nothing; sum_j dK_j = 0 (the softmax is shift
      invariant in the scores) and sum_j dV_j = sum_i dout_i (each query's probabilities sum to 1)
  X4  a sample without keys: out = 0, lse = -inf, zero gradients; without queries: nothing written, dk = dv = 0
"""
import numpy as np
import pytest
import torch

from oracle import cross


def _data(Lq, Lk, H, D, seed=0):
    rng = np.random.default_rng(seed)
    oq = np.concatenate([[0], np.cumsum(Lq)]); ok = np.concatenate([[0], np.cumsum(Lk)])
    mk = lambda n: rng.standard_normal((n, H, D))
    return mk(oq[-1]), mk(ok[-1]), mk(ok[-1]), mk(oq[-1]), oq, ok


def test_x1_equal_offsets_is_the_c_oracle(oracle):
    L = [7, 1, 0, 12, 3]
    q, k, v, do, oq, _ = _data(L, L, 2, 8, seed=1)
    q, k, v, do = (a.astype(np.float32) for a in (q, k, v, do))
    out_c, lse_c = oracle.forward(q, k, v, oq)
    out_x, lse_x = cross.forward(q, k, v, oq, oq)
    np.testing.assert_allclose(out_x, out_c, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse_x, lse_c, rtol=1e-12, atol=1e-13)
    ref = oracle.backward(q, k, v, do, oq)
    got = cross.backward(q, k, v, do, oq, oq)
    for g, r in zip(got, ref):
        np.testing.assert_allclose(g, r, rtol=1e-11, atol=1e-12)


def test_x2_torch_sdpa_with_different_lengths():
    Lq, Lk = [5, 2, 9, 1], [3, 11, 4, 6]
    q, k, v, do, oq, ok = _data(Lq, Lk, 2, 4, seed=2)
    qt, kt, vt = (torch.from_numpy(a).requires_grad_(True) for a in (q, k, v))
    outs = []
    for b in range(len(Lq)):
        a = [x[o[b]:o[b + 1]].transpose(0, 1) for x, o in ((qt, oq), (kt, ok), (vt, ok))]     # [H, L, D]
        outs.append(torch.nn.functional.scaled_dot_product_attention(*a).transpose(0, 1))
    out_t = torch.cat(outs)
    (out_t * torch.from_numpy(do)).sum().backward()
    out, lse = cross.forward(q, k, v, oq, ok)
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-12, atol=1e-13)
    dq, dk, dv, delta = cross.backward(q, k, v, do, oq, ok)
    np.testing.assert_allclose(dq, qt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dk, kt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dv, vt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(delta, (do * out).sum(axis=2).T, rtol=1e-12, atol=1e-13)
    s = np.einsum("hd,jhd->hj", q[0], k[:3]) / 2.0                                            # lse of the first query row
    np.testing.assert_allclose(lse[:, 0], np.log(np.exp(s).sum(axis=1)), rtol=1e-13)


def test_x3_closed_forms():
    q, k, v, _, oq, ok = _data([4, 3], [1, 5], 2, 8, seed=3)
    out, lse = cross.forward(q, k, v, oq, ok)
    np.testing.assert_allclose(out[:4], np.broadcast_to(v[0], (4, 2, 8)), rtol=1e-15)           # one key: its value row
    np.testing.assert_allclose(lse[:, :4], np.einsum("ihd,hd->hi", q[:4], k[0]) / np.sqrt(8), rtol=1e-14)
    k2 = k.copy(); k2[1:] = k[1]                                                               # equal keys: mean of the values
    out2, lse2 = cross.forward(q, k2, v, oq, ok)
    np.testing.assert_allclose(out2[4:], np.broadcast_to(v[1:].mean(axis=0), (3, 2, 8)), rtol=1e-13)
    np.testing.assert_allclose(lse2[:, 4:], np.einsum("ihd,hd->hi", q[4:], k[1]) / np.sqrt(8) + np.log(5), rtol=1e-13)
    perm = np.array([0, 3, 1, 5, 2, 4])                                                        # permute sample 1's keys
    out3, lse3 = cross.forward(q, k[perm], v[perm], oq, ok)
    np.testing.assert_allclose(out3, out, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse3, lse, rtol=1e-13)
    dq, dk, dv, _ = cross.backward(q, k, v, np.ones_like(q), oq, ok)
    np.testing.assert_allclose(dk[1:].sum(axis=0), 0.0, atol=1e-13)                             # softmax is shift invariant in the scores
    np.testing.assert_allclose(dv[1:].sum(axis=0), 3.0, rtol=1e-13)                             # each query's probabilities sum to 1


def test_x4_empty_sides():
    q, k, v, do, oq, ok = _data([3, 0, 2], [0, 4, 5], 1, 4, seed=4)
    out, lse = cross.forward(q, k, v, oq, ok)
    assert (out[:3] == 0).all() and np.isneginf(lse[:, :3]).all() and np.isfinite(lse[:, 3:]).all()
    dq, dk, dv, delta = cross.backward(q, k, v, do, oq, ok)
    assert (dq[:3] == 0).all() and (dk[:4] == 0).all() and (dv[:4] == 0).all() and (delta[:, :3] == 0).all()
    assert np.abs(dk[4:]).max() > 0
