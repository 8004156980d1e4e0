"""Pins for the CPU oracle: each test checks oracle/jfa_oracle.c against something that is NOT the oracle.

  P1  brute-force padded dense attention with key masking, written in numpy (the paper's comparison
      system "dense attention with padding", Section 3 / Table 1 caption)
  P2  equal-length batches reduce to torch's fp64 scaled_dot_product_attention, and its autograd
      gives dQ, dK, dV
  P3  the unfused three-step formulation of Table 1 (scores as a [sum Bi*Bi] array, jagged2 softmax,
      array x jagged product)
  P4  softmax rows sum to one; sum_j exp(S_ij - LSE_i) = 1
  P5  a length-1 sample returns its own V row, lse = q.k/sqrt(D), dV = dO, dQ = dK = 0
  P6  permuting the samples permutes the results
  P7  closed forms: equal keys or zero queries give the mean of V and lse = S + ln L
  P8  shift invariance and gradient identities
  P9  central finite differences of sum(out * dO)
  P10 large scores stay finite; a row whose scores are all far below zero keeps its softmax (the maximum is
      subtracted before the exponentials, not zero)
  P11 rows past offsets[B] are never read
"""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom, make_workload, offsets_from_lengths


def dense_padded_attention(q, k, v, offsets):
    """Numpy fp64: scatter to [B, Lmax, H, D] zero padded, mask keys >= L_b with -inf, gather valid rows."""
    offsets = np.asarray(offsets)
    B = len(offsets) - 1
    lens = np.diff(offsets)
    _, H, D = q.shape
    Lmax = max(int(lens.max()), 1)
    qd = np.zeros((B, Lmax, H, D)); kd = np.zeros_like(qd); vd = np.zeros_like(qd)
    for b in range(B):
        s, L = offsets[b], lens[b]
        qd[b, :L] = q[s:s + L]; kd[b, :L] = k[s:s + L]; vd[b, :L] = v[s:s + L]
    S = np.einsum("bihd,bjhd->bhij", qd, kd) / np.sqrt(D)
    mask = np.arange(Lmax)[None, :] >= lens[:, None]            # [B, Lmax] True where padded
    S = np.where(mask[:, None, None, :], -np.inf, S)
    with np.errstate(invalid="ignore"):                         # rows of zero-length samples are all -inf
        m = S.max(axis=-1, keepdims=True)
        E = np.exp(S - m)
        l = E.sum(axis=-1, keepdims=True)
        O = np.einsum("bhij,bjhd->bihd", E / l, vd)
        lse_d = (m + np.log(l))[..., 0]                         # [B, H, Lmax]
    out = np.zeros((int(offsets[-1]), H, D)); lse = np.zeros((H, int(offsets[-1])))
    for b in range(B):
        s, L = offsets[b], lens[b]
        out[s:s + L] = O[b, :L]
        lse[:, s:s + L] = lse_d[b, :, :L]
    return out, lse


@pytest.mark.parametrize("seed,lengths,H,D", [
    (0, [5, 1, 17, 3], 2, 8), (1, [1, 1, 1], 1, 4), (2, [9, 0, 4, 0, 12, 7], 3, 4), (3, [16], 1, 8),
])
def test_p1_padded_dense_bruteforce(oracle, seed, lengths, H, D):
    w = make_custom("t", lengths, H, D, dtype="f32", seed=seed)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    ref_out, ref_lse = dense_padded_attention(w.q.astype(np.float64), w.k.astype(np.float64),
                                              w.v.astype(np.float64), w.offsets)
    np.testing.assert_allclose(out, ref_out, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("B,L,H,D", [(3, 11, 2, 8), (2, 33, 3, 16)])
def test_p2_equal_lengths_match_torch_sdpa_and_autograd(oracle, B, L, H, D):
    w = make_custom("t", [L] * B, H, D, dtype="f32", seed=7)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    dq, dk, dv, delta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)

    def to_bhld(x):
        return torch.from_numpy(x.astype(np.float64)).reshape(B, L, H, D).permute(0, 2, 1, 3).contiguous()

    tq, tk, tv = (to_bhld(x).requires_grad_(True) for x in (w.q, w.k, w.v))
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)          # default scale 1/sqrt(D), non-causal
    to.backward(to_bhld(w.dout))

    def back(t):
        return t.detach().permute(0, 2, 1, 3).reshape(B * L, H, D).numpy()

    np.testing.assert_allclose(out, back(to), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dq, back(tq.grad), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, back(tk.grad), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, back(tv.grad), rtol=1e-10, atol=1e-12)
    # lse against torch.logsumexp of the scaled scores
    S = torch.einsum("bhid,bhjd->bhij", tq.detach(), tk.detach()) / np.sqrt(D)
    ref_lse = torch.logsumexp(S, dim=-1).permute(1, 0, 2).reshape(H, B * L).numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(delta, np.einsum("nhd,nhd->hn", w.dout.astype(np.float64), out), rtol=1e-11, atol=1e-12)


def test_p2b_jagged_backward_matches_per_sample_autograd(oracle):
    """Ragged lengths: run torch autograd sample by sample (no padding involved)."""
    w = make_custom("t", [7, 1, 13, 4], 2, 8, dtype="f32", seed=11)
    dq, dk, dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    for b in range(w.B):
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        ts = [torch.from_numpy(x[s:e].astype(np.float64)).permute(1, 0, 2).contiguous().requires_grad_(True)
              for x in (w.q, w.k, w.v)]
        o = torch.softmax(ts[0] @ ts[1].transpose(1, 2) / np.sqrt(w.D), dim=-1) @ ts[2]
        o.backward(torch.from_numpy(w.dout[s:e].astype(np.float64)).permute(1, 0, 2))
        for got, t in zip((dq, dk, dv), ts):
            np.testing.assert_allclose(got[s:e], t.grad.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_p3_unfused_three_step_formulation(oracle):
    """Table 1: jagged x jagged -> [sum Bi*Bi]; softmax over each row segment; array x jagged -> [sum_B, D]."""
    w = make_custom("t", [6, 2, 9], 2, 4, dtype="f32", seed=5)
    out, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    q, k, v = (x.astype(np.float64) for x in (w.q, w.k, w.v))
    sq_off = offsets_from_lengths(w.lengths ** 2)
    for h in range(w.H):
        scores = np.zeros(int(sq_off[-1]))
        for b in range(w.B):                                   # step 1
            s, L = int(w.offsets[b]), int(w.lengths[b])
            for i in range(L):
                for j in range(L):
                    scores[sq_off[b] + i * L + j] = q[s + i, h] @ k[s + j, h] / np.sqrt(w.D)
        for b in range(w.B):                                   # step 2
            L = int(w.lengths[b])
            for i in range(L):
                seg = scores[sq_off[b] + i * L: sq_off[b] + (i + 1) * L]
                e = np.exp(seg - seg.max())
                seg[:] = e / e.sum()
        for b in range(w.B):                                   # step 3
            s, L = int(w.offsets[b]), int(w.lengths[b])
            for i in range(L):
                o = sum(scores[sq_off[b] + i * L + j] * v[s + j, h] for j in range(L))
                np.testing.assert_allclose(out[s + i, h], o, rtol=1e-12, atol=1e-13)


def test_p4_softmax_rows_sum_to_one_and_lse_convention(oracle):
    w = make_custom("t", [8, 3, 15], 2, 8, dtype="f32", seed=3)
    _, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    for b in range(w.B):
        s, L = int(w.offsets[b]), int(w.lengths[b])
        for h in range(w.H):
            P = oracle.probs(w.q, w.k, w.v, w.offsets, b, h)
            assert P.shape == (L, L) and (P >= 0).all()
            np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)
            S = w.q[s:s + L, h].astype(np.float64) @ w.k[s:s + L, h].astype(np.float64).T / np.sqrt(w.D)
            np.testing.assert_allclose(np.exp(S - lse[h, s:s + L, None]).sum(axis=1), 1.0, rtol=0, atol=1e-13)
            np.testing.assert_allclose(np.exp(S - lse[h, s:s + L, None]), P, rtol=1e-12, atol=1e-15)


def test_p5_length_one_sample(oracle):
    w = make_custom("t", [4, 1, 6, 1], 2, 8, dtype="f32", seed=9)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    dq, dk, dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    for b in (1, 3):
        s = int(w.offsets[b])
        np.testing.assert_array_equal(out[s], w.v[s].astype(np.float64))
        np.testing.assert_allclose(lse[:, s], np.einsum("hd,hd->h", w.q[s].astype(np.float64),
                                                        w.k[s].astype(np.float64)) / np.sqrt(w.D), rtol=1e-14)
        np.testing.assert_array_equal(dv[s], w.dout[s].astype(np.float64))
        np.testing.assert_allclose(dq[s], 0.0, atol=1e-15)
        np.testing.assert_allclose(dk[s], 0.0, atol=1e-15)


def test_p6_sample_permutation_invariance(oracle):
    w = make_custom("t", [5, 12, 1, 8, 3], 2, 8, dtype="f32", seed=13)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    dq, dk, dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    perm = [3, 0, 4, 2, 1]
    rows = np.concatenate([np.arange(w.offsets[b], w.offsets[b + 1]) for b in perm])
    off2 = offsets_from_lengths(w.lengths[perm])
    out2, lse2 = oracle.forward(w.q[rows], w.k[rows], w.v[rows], off2)
    dq2, dk2, dv2, _ = oracle.backward(w.q[rows], w.k[rows], w.v[rows], w.dout[rows], off2)
    np.testing.assert_array_equal(out2, out[rows])
    np.testing.assert_array_equal(lse2, lse[:, rows])
    np.testing.assert_array_equal(dq2, dq[rows])
    np.testing.assert_array_equal(dk2, dk[rows])
    np.testing.assert_array_equal(dv2, dv[rows])


def test_p7_closed_forms_uniform_attention(oracle):
    w = make_custom("t", [7, 10], 2, 8, dtype="f32", seed=17)
    # (a) all keys of a sample equal -> uniform weights
    k = w.k.copy()
    for b in range(w.B):
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        k[s:e] = k[s]
    out, lse = oracle.forward(w.q, k, w.v, w.offsets)
    for b in range(w.B):
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        mean_v = w.v[s:e].astype(np.float64).mean(axis=0)
        np.testing.assert_allclose(out[s:e], np.broadcast_to(mean_v, (e - s,) + mean_v.shape), rtol=1e-13, atol=1e-14)
        s0 = np.einsum("ihd,hd->hi", w.q[s:e].astype(np.float64), k[s].astype(np.float64)) / np.sqrt(w.D)
        np.testing.assert_allclose(lse[:, s:e], s0 + np.log(e - s), rtol=1e-13, atol=1e-14)
    # (b) zero queries -> the same, with lse = ln L
    out, lse = oracle.forward(np.zeros_like(w.q), w.k, w.v, w.offsets)
    for b in range(w.B):
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        np.testing.assert_allclose(out[s:e], np.broadcast_to(w.v[s:e].astype(np.float64).mean(axis=0), out[s:e].shape),
                                   rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(lse[:, s:e], np.log(e - s), rtol=1e-14)


def test_p8_shift_invariance_and_gradient_identities(oracle):
    w = make_custom("t", [9, 4, 14], 2, 8, dtype="f32", seed=19)
    out, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    # q_i . (k_j + c) = q_i . k_j + q_i . c: a per-row constant, removed by the softmax.
    # Use a shift exactly representable in fp32 sums so the inputs stay exact.
    k2 = w.k.copy()
    shift = np.zeros((w.H, w.D), dtype=np.float32); shift[:, ::2] = 0.5; shift[:, 1::2] = -0.25
    k2 = (k2.astype(np.float64) + shift).astype(np.float32)
    out2, _ = oracle.forward(w.q, k2, w.v, w.offsets)
    np.testing.assert_allclose(out2, out, rtol=0, atol=2e-6)     # fp32 re-rounding of k + c only
    dq, dk, dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    for b in range(w.B):
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        # rows of dS sum to zero, and dK_j = scale sum_i dS_ij Q_i, so
        # sum_j dK_j = scale sum_i Q_i (sum_j dS_ij) = 0.
        np.testing.assert_allclose(dk[s:e].sum(axis=0), 0.0, atol=1e-12)
        # columns: sum_j dV_j = sum_i (sum_j P_ij) dO_i = sum_i dO_i
        np.testing.assert_allclose(dv[s:e].sum(axis=0), w.dout[s:e].astype(np.float64).sum(axis=0), rtol=1e-12, atol=1e-12)


def test_p9_finite_differences(oracle):
    w = make_custom("t", [6, 3, 10], 2, 4, dtype="f32", seed=23)
    dq, dk, dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    rng = np.random.default_rng(0)
    # fp32 inputs: step by an exactly representable 2^-7 and rely on fp64 evaluation inside the oracle
    h = 2.0 ** -7

    def loss(q, k, v):
        out, _ = oracle.forward(q, k, v, w.offsets)
        return float((out * w.dout.astype(np.float64)).sum())

    # Richardson-extrapolated central difference (error O(h^4)) so a coarse, exactly representable step suffices
    for name, grad in (("q", dq), ("k", dk), ("v", dv)):
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in w.q.shape)
            vals = []
            for step in (h, h / 2):
                args = {"q": w.q.copy(), "k": w.k.copy(), "v": w.v.copy()}
                base = float(args[name][idx])
                # keep the perturbed value exactly representable in fp32
                args[name][idx] = np.float32(base + step); up = loss(**args); du = float(args[name][idx]) - base
                args[name][idx] = np.float32(base - step); dn = loss(**args); dd = base - float(args[name][idx])
                assert du == step and dd == step
                vals.append((up - dn) / (2 * step))
            fd = (4 * vals[1] - vals[0]) / 3
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])


def test_p10_large_scores_are_stable(oracle):
    w = make_custom("t", [12, 5], 2, 8, dtype="f32", seed=29)
    q = (w.q * np.float32(64.0)).astype(np.float32)               # scores of order +-hundreds
    out, lse = oracle.forward(q, w.k, w.v, w.offsets)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    ref_out, ref_lse = dense_padded_attention(q.astype(np.float64), w.k.astype(np.float64), w.v.astype(np.float64), w.offsets)
    np.testing.assert_allclose(out, ref_out, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12)
    dq, dk, dv, _ = oracle.backward(q, w.k, w.v, w.dout, w.offsets)
    assert all(np.isfinite(g).all() for g in (dq, dk, dv))


def test_p10b_rows_with_only_very_negative_scores(oracle):
    """Every score of every row lies below -800 (queries are positive multiples of one direction, keys negative
    multiples of it): exp(score) underflows to zero in fp64, so the softmax only exists if the row maximum is
    subtracted first.  Expected values from scipy's logsumexp / softmax on the same fp64 scores."""
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(41)
    lengths, H, D = [7, 1, 4], 2, 8
    off = offsets_from_lengths(np.asarray(lengths))
    n = int(off[-1])
    u = rng.standard_normal((H, D)).astype(np.float32)
    a = rng.uniform(20.0, 30.0, size=(n, H, 1)).astype(np.float32)
    b = rng.uniform(20.0, 30.0, size=(n, H, 1)).astype(np.float32)
    q = (a * u[None]).astype(np.float32)
    k = (-b * u[None]).astype(np.float32)
    v = rng.standard_normal((n, H, D)).astype(np.float32)
    dout = rng.standard_normal((n, H, D)).astype(np.float32)
    out, lse = oracle.forward(q, k, v, off)
    dq, dk, dv, _ = oracle.backward(q, k, v, dout, off)
    assert all(np.isfinite(x).all() for x in (out, lse, dq, dk, dv))
    for bidx, L in enumerate(lengths):
        s = int(off[bidx])
        for h in range(H):
            S = q[s:s + L, h].astype(np.float64) @ k[s:s + L, h].astype(np.float64).T / np.sqrt(D)
            assert S.max() < -800.0
            np.testing.assert_allclose(lse[h, s:s + L], logsumexp(S, axis=1), rtol=1e-13)
            P = softmax(S, axis=1)
            np.testing.assert_allclose(out[s:s + L, h], P @ v[s:s + L, h].astype(np.float64), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(dv[s:s + L, h], P.T @ dout[s:s + L, h].astype(np.float64), rtol=1e-10, atol=1e-12)


def test_p11_rows_past_the_last_offset_are_ignored(oracle):
    w = make_custom("t", [5, 8], 2, 8, dtype="f32", seed=31)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    pad = np.full((3, w.H, w.D), np.nan, dtype=np.float32)
    out2, lse2 = oracle.forward(np.concatenate([w.q, pad]), np.concatenate([w.k, pad]), np.concatenate([w.v, pad]), w.offsets)
    np.testing.assert_array_equal(out2, out)
    np.testing.assert_array_equal(lse2, lse)


def test_pairs_subset_equals_full(oracle):
    w = make_custom("t", [5, 8, 3], 2, 8, dtype="f32", seed=37)
    out, lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    out2, lse2 = oracle.forward(w.q, w.k, w.v, w.offsets, pairs=[(1, 0), (2, 1)])
    s, e = int(w.offsets[1]), int(w.offsets[2])
    np.testing.assert_array_equal(out2[s:e, 0], out[s:e, 0])
    np.testing.assert_array_equal(lse2[0, s:e], lse[0, s:e])
    assert np.isnan(out2[s:e, 1]).all() and np.isnan(out2[: int(w.offsets[1])]).all()
    s, e = int(w.offsets[2]), int(w.offsets[3])
    np.testing.assert_array_equal(out2[s:e, 1], out[s:e, 1])


def test_bf16_workload_values_are_bf16_representable():
    w = make_workload("c2_geom_bf16")
    assert w.sum_B == 14848 and w.S2 == 1527456
    u = w.q.view(np.uint32)
    assert (u & 0xFFFF == 0).all()
    assert (w.bits["q"].astype(np.uint32) << 16 == u).all()
