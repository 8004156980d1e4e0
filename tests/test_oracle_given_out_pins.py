"""Pins for oracle/given_out.py (the backward with delta formed from a given output tensor).

  G1  given the exact fp64 output it is the plain backward: equal to oracle/jfa_oracle.c, and under the mask to
      oracle/causal.py, which are pinned on their own (torch autograd, finite differences)
  G2  delta is the row sum of dout * (given out), whatever out is
  G3  a perturbation e of out moves dq by exactly -(1/sqrt(D)) (sum_j P_ij k_j) (dout_i . e_i): checked in closed form
      on a sample of length 1 (P = 1: dq = (dout.v - dout.out) k / sqrt(D))
"""
import numpy as np

from oracle import causal as causal_oracle, given_out
from paper_2409_15373_amd.synthetic import make_custom


def test_g1_exact_output_gives_the_plain_backward(oracle):
    w = make_custom("t", [7, 0, 1, 12, 3], 2, 8, dtype="f32", seed=51)
    out, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    ref = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    got = given_out.backward(w.q, w.k, w.v, out, w.dout, w.offsets)
    for g, r in zip(got, ref):
        np.testing.assert_allclose(g, r, rtol=1e-11, atol=1e-12)
    out_c, _ = causal_oracle.forward(w.q, w.k, w.v, w.offsets)
    ref_c = causal_oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    got_c = given_out.backward(w.q, w.k, w.v, out_c, w.dout, w.offsets, causal=True)
    for g, r in zip(got_c, ref_c):
        np.testing.assert_allclose(g, r, rtol=1e-11, atol=1e-12)


def test_g2_delta_is_the_row_sum_of_the_given_output():
    w = make_custom("t", [5, 9], 3, 4, dtype="f32", seed=52)
    fake_out = np.random.default_rng(1).standard_normal(w.q.shape)
    *_, delta = given_out.backward(w.q, w.k, w.v, fake_out, w.dout, w.offsets)
    np.testing.assert_allclose(delta, (w.dout.astype(np.float64) * fake_out).sum(-1).T, rtol=1e-13)


def test_g3_length_one_closed_form():
    w = make_custom("t", [1, 1, 1], 2, 8, dtype="f32", seed=53)
    fake_out = np.random.default_rng(2).standard_normal(w.q.shape)
    dq, dk, dv, _ = given_out.backward(w.q, w.k, w.v, fake_out, w.dout, w.offsets)
    q, k, v, do = (x.astype(np.float64) for x in (w.q, w.k, w.v, w.dout))
    ds = ((do * v).sum(-1) - (do * fake_out).sum(-1))[..., None]          # P = 1
    np.testing.assert_allclose(dq, ds * k / np.sqrt(8), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dk, ds * q / np.sqrt(8), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dv, do, rtol=0, atol=0)
