"""Pins for oracle/unfused.py (the three separate operators of the paper's unfused "jagged attention", Table 1):
each test checks it against something that is not itself.

  U1  scores / softmax_rows / apply against torch fp64 per sample (matmul, torch.softmax)
  U2  their composition equals the attention forward of the C oracle (another program, another language)
  U3  closed forms: q = k gives symmetric score blocks with |k_i|^2 / sqrt(D) on the diagonal; constant
      score rows give uniform probabilities; an identity probability block returns V
  U4  layout: the score of (sample b, head h, query i, key j) sits at [h, sq[b] + i * L_b + j]; zero-length
      samples take no room; nothing of one sample reaches another
  U5  backward operators: product(q, k, 1/sqrt(D)) is scores; the chain dP = product(dout, v, 1),
      dS = softmax_rows_backward(P, dP, 1/sqrt(D)), dV = apply_transposed(P, dout), dQ = apply(dS, k),
      dK = apply_transposed(dS, q) equals the backward of the C attention oracle and torch autograd through the
      unfused forward; softmax_rows_backward is the vector-Jacobian product of torch.softmax row by row
"""
import numpy as np
import pytest
import torch

from oracle import unfused
from paper_2409_15373_amd.synthetic import make_custom


def _workload(lengths, H, D, seed=0):
    return make_custom("unfused", lengths, H, D, "f32", sigma=1.0, seed=seed)


@pytest.mark.parametrize("lengths,H,D", [([5, 1, 0, 9, 3], 2, 8), ([17, 4], 3, 4)])
def test_u1_each_step_matches_torch(lengths, H, D):
    w = _workload(lengths, H, D)
    S = unfused.scores(w.q, w.k, w.offsets)
    P = unfused.softmax_rows(S, w.offsets)
    out = unfused.apply(P, w.v, w.offsets)
    sq = unfused.square_offsets(w.offsets)
    q, k, v = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (w.q, w.k, w.v))
    for b, L in enumerate(lengths):
        s = int(w.offsets[b])
        for h in range(H):
            St = (q[s:s + L, h] @ k[s:s + L, h].T) / D ** 0.5
            Pt = torch.softmax(St, dim=-1)
            np.testing.assert_allclose(S[h, sq[b]:sq[b + 1]].reshape(L, L), St.numpy(), rtol=1e-13, atol=1e-13)
            np.testing.assert_allclose(P[h, sq[b]:sq[b + 1]].reshape(L, L), Pt.numpy(), rtol=1e-13, atol=1e-15)
            np.testing.assert_allclose(out[s:s + L, h], (Pt @ v[s:s + L, h]).numpy(), rtol=1e-12, atol=1e-13)


def test_u2_composition_equals_the_attention_oracle(oracle):
    w = _workload([33, 1, 7, 0, 20], 2, 16, seed=3)
    out_c, lse_c = oracle.forward(w.q, w.k, w.v, w.offsets)
    S = unfused.scores(w.q, w.k, w.offsets)
    out_u = unfused.apply(unfused.softmax_rows(S, w.offsets), w.v, w.offsets)
    np.testing.assert_allclose(out_u, out_c, rtol=1e-11, atol=1e-12)
    sq = unfused.square_offsets(w.offsets)                      # and the log-sum-exp of the score rows
    for b in range(len(w.offsets) - 1):
        L = int(w.offsets[b + 1] - w.offsets[b])
        s = int(w.offsets[b])
        for h in range(w.H):
            blk = S[h, sq[b]:sq[b + 1]].reshape(L, L)
            if L:
                m = blk.max(axis=1)
                np.testing.assert_allclose(m + np.log(np.exp(blk - m[:, None]).sum(axis=1)), lse_c[h, s:s + L],
                                           rtol=1e-12, atol=1e-12)


def test_u3_closed_forms():
    w = _workload([6, 4], 2, 8, seed=1)
    sq = unfused.square_offsets(w.offsets)
    S = unfused.scores(w.k, w.k, w.offsets)                      # q = k: symmetric blocks, squared norms on the diagonal
    for b in range(2):
        L = int(w.offsets[b + 1] - w.offsets[b]); s = int(w.offsets[b])
        for h in range(2):
            blk = S[h, sq[b]:sq[b + 1]].reshape(L, L)
            np.testing.assert_allclose(blk, blk.T, rtol=0, atol=1e-15)
            kk = np.asarray(w.k, dtype=np.float64)[s:s + L, h]
            np.testing.assert_allclose(np.diag(blk), (kk * kk).sum(axis=1) / np.sqrt(8), rtol=1e-14)
    const = np.full((2, int(sq[-1])), 3.25)                      # constant rows: uniform probabilities
    P = unfused.softmax_rows(const, w.offsets)
    np.testing.assert_allclose(P[:, :36], 1 / 6, rtol=1e-15)
    np.testing.assert_allclose(P[:, 36:], 1 / 4, rtol=1e-15)
    eye = np.zeros((2, int(sq[-1])))                             # identity blocks: apply returns V
    eye[:, :36] = np.eye(6).reshape(36); eye[:, 36:] = np.eye(4).reshape(16)
    np.testing.assert_array_equal(unfused.apply(eye, w.v, w.offsets), np.asarray(w.v, dtype=np.float64))


def test_u4_layout_and_sample_isolation():
    w = _workload([3, 0, 2], 2, 4, seed=2)
    sq = unfused.square_offsets(w.offsets)
    assert sq.tolist() == [0, 9, 9, 13]
    S = unfused.scores(w.q, w.k, w.offsets)
    assert S.shape == (2, 13)
    q = np.asarray(w.q, dtype=np.float64); k = np.asarray(w.k, dtype=np.float64)
    assert S[1, 0 * 3 + 2] == pytest.approx(q[0, 1] @ k[2, 1] / 2.0, rel=1e-14)            # b=0, h=1, i=0, j=2
    assert S[0, 9 + 1 * 2 + 0] == pytest.approx(q[3 + 1, 0] @ k[3 + 0, 0] / 2.0, rel=1e-14)  # b=2, h=0, i=1, j=0
    k2 = k.copy(); k2[3:] = 7.0                                   # change sample 2 only: sample 0's scores stay
    S2 = unfused.scores(q, k2, w.offsets)
    np.testing.assert_array_equal(S2[:, :9], S[:, :9])
    assert not np.array_equal(S2[:, 9:], S[:, 9:])


def test_u5_backward_chain(oracle):
    w = make_custom("unfused", [9, 1, 0, 14, 4], 2, 8, "f32", sigma=1.0, seed=5)
    q, k, v, do = (np.asarray(x, dtype=np.float64) for x in (w.q, w.k, w.v, w.dout))
    c = 1.0 / np.sqrt(8)
    np.testing.assert_allclose(unfused.product(q, k, w.offsets, c), unfused.scores(q, k, w.offsets), rtol=1e-14, atol=1e-15)   # x * c vs x / sqrt(D)
    P = unfused.softmax_rows(unfused.scores(q, k, w.offsets), w.offsets)
    dP = unfused.product(do, v, w.offsets, 1.0)
    dS = unfused.softmax_rows_backward(P, dP, w.offsets, c)
    dV, dQ, dK = unfused.apply_transposed(P, do, w.offsets), unfused.apply(dS, k, w.offsets), unfused.apply_transposed(dS, q, w.offsets)
    r_dq, r_dk, r_dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)        # the C oracle: another program
    np.testing.assert_allclose(dQ, r_dq, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, r_dk, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, r_dv, rtol=1e-10, atol=1e-12)
    # softmax_rows_backward against autograd of torch.softmax, one block
    sq = unfused.square_offsets(w.offsets)
    S = torch.from_numpy(unfused.scores(q, k, w.offsets)[1, sq[3]:sq[4]].reshape(14, 14)).requires_grad_(True)
    g = torch.from_numpy(dP[1, sq[3]:sq[4]].reshape(14, 14))
    (torch.softmax(S, dim=1) * g).sum().backward()
    np.testing.assert_allclose(unfused.softmax_rows_backward(P, dP, w.offsets)[1, sq[3]:sq[4]].reshape(14, 14), S.grad.numpy(),
                               rtol=1e-11, atol=1e-13)
