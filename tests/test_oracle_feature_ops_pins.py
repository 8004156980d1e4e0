"""Pins for oracle/feature_ops.py (Table 1's jagged_dense_bmm, jagged_jagged_bmm, jagged_softmax), each against
something that is not the oracle's own line:

  F1  padded formulation in torch fp64: torch.bmm on zero-padded dense tensors (the paper's "PyTorch version"),
      and a -inf-padded torch.softmax along the length axis
  F2  autograd: jagged_jagged_bmm is the gradient of sum(jagged_dense_bmm * g) with respect to w, jagged_dense_bmm
      with w transposed the gradient with respect to x; jagged_softmax_backward is the vector-Jacobian product
      of torch.softmax per sample
  F3  closed forms and invariants: identity w returns x; columns of the softmax sum to 1 per sample, are uniform
      for constant columns, and do not change when a per-column constant is added; the backward of a constant dy is 0
  F4  hand case, empty samples, sample isolation
"""
import numpy as np
import pytest
import torch

from oracle import feature_ops as fo
from paper_2409_15373_amd.synthetic import offsets_from_lengths

LENGTHS = np.array([5, 0, 9, 1, 3])


def _data(D, T, seed=0):
    rng = np.random.default_rng(seed)
    off = offsets_from_lengths(LENGTHS)
    n = int(off[-1])
    return off, rng.standard_normal((n, D)), rng.standard_normal((n, T)), rng.standard_normal((len(LENGTHS), D, T))


def _pad(a, off, N, fill=0.0):
    B = len(off) - 1
    d = np.full((B, N) + a.shape[1:], fill)
    for b in range(B):
        d[b, :off[b + 1] - off[b]] = a[off[b]:off[b + 1]]
    return torch.from_numpy(d)


def test_f1_padded_torch_formulation():
    off, x, y, w = _data(6, 4)
    N = 9
    xp, yp = _pad(x, off, N), _pad(y, off, N)
    ref = torch.bmm(xp, torch.from_numpy(w)).numpy()                        # [B, N, T]
    got = fo.jagged_dense_bmm(x, w, off)
    for b, L in enumerate(LENGTHS):
        np.testing.assert_allclose(got[off[b]:off[b + 1]], ref[b, :L], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(fo.jagged_jagged_bmm(x, y, off), torch.bmm(xp.transpose(1, 2), yp).numpy(), rtol=1e-13, atol=1e-13)
    sm = torch.softmax(_pad(x, off, N, fill=-np.inf), dim=1).numpy()          # along the length axis; empty sample: nan, unused
    got = fo.jagged_softmax(x, off)
    for b, L in enumerate(LENGTHS):
        np.testing.assert_allclose(got[off[b]:off[b + 1]], sm[b, :L], rtol=1e-13, atol=1e-15)


def test_f2_gradients_by_autograd():
    off, x, g, w = _data(5, 3, seed=1)                                      # g plays the output's gradient [n, T]
    xt = torch.from_numpy(x).requires_grad_(True)
    wt = torch.from_numpy(w).requires_grad_(True)
    out = torch.cat([xt[off[b]:off[b + 1]] @ wt[b] for b in range(len(LENGTHS))])
    (out * torch.from_numpy(g)).sum().backward()
    np.testing.assert_allclose(fo.jagged_jagged_bmm(x, g, off), wt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(fo.jagged_dense_bmm(g, np.transpose(w, (0, 2, 1)), off), xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    dy = np.random.default_rng(2).standard_normal(x.shape)
    xt = torch.from_numpy(x).requires_grad_(True)
    y = torch.cat([torch.softmax(xt[off[b]:off[b + 1]], dim=0) for b in range(len(LENGTHS)) if LENGTHS[b]])
    (y * torch.from_numpy(dy)).sum().backward()
    np.testing.assert_allclose(fo.jagged_softmax_backward(fo.jagged_softmax(x, off), dy, off), xt.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_f3_closed_forms():
    off, x, _, _ = _data(4, 4, seed=3)
    eye = np.broadcast_to(np.eye(4), (len(LENGTHS), 4, 4))
    np.testing.assert_array_equal(fo.jagged_dense_bmm(x, eye, off), x)
    y = fo.jagged_softmax(x, off)
    for b, L in enumerate(LENGTHS):
        if L:
            np.testing.assert_allclose(y[off[b]:off[b + 1]].sum(axis=0), 1.0, rtol=1e-14)
    np.testing.assert_allclose(fo.jagged_softmax(x + np.array([3.0, -2.0, 100.0, 0.5]), off), y, rtol=1e-12)
    c = np.tile(np.array([1.0, -4.0, 0.0, 7.0]), (x.shape[0], 1))
    yc = fo.jagged_softmax(c, off)
    for b, L in enumerate(LENGTHS):
        if L:
            np.testing.assert_allclose(yc[off[b]:off[b + 1]], 1.0 / L, rtol=1e-14)
    np.testing.assert_allclose(fo.jagged_softmax_backward(y, np.full_like(y, 2.5), off), 0.0, atol=1e-15)


def test_f4_hand_case_and_isolation():
    off = np.array([0, 2, 2, 3])
    x = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    w = np.array([[[1.0], [1.0]], [[9.0], [9.0]], [[2.0], [-1.0]]])           # [B = 3, D = 2, T = 1]
    assert fo.jagged_dense_bmm(x, w, off).ravel().tolist() == [3.0, 7.0, 4.0]
    yv = np.array([[1.0], [2.0], [3.0]])
    assert fo.jagged_jagged_bmm(x, yv, off).tolist() == [[[7.0], [10.0]], [[0.0], [0.0]], [[15.0], [18.0]]]
    sm = fo.jagged_softmax(x, off)
    e = np.exp(-2.0)
    np.testing.assert_allclose(sm, [[e / (1 + e)] * 2, [1 / (1 + e)] * 2, [1.0, 1.0]], rtol=1e-14)
    x2 = x.copy(); x2[2] = -50.0                                             # change sample 2 only
    np.testing.assert_array_equal(fo.jagged_softmax(x2, off)[:2], sm[:2])
    np.testing.assert_array_equal(fo.jagged_jagged_bmm(x2, yv, off)[0], fo.jagged_jagged_bmm(x, yv, off)[0])
