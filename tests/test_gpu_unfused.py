"""The unfused jagged attention operators (Table 1) on the GPU vs oracle/unfused.py on the same seeded bf16 inputs.

  square offsets  bit exact (integers)
  scores          fp32 products of bf16 inputs with fp32 accumulation: |gpu - oracle| <= 1e-4 * max(1, |oracle|)
  softmax         fed with the GPU's own scores: |gpu - oracle(softmax of those scores)| <= 2e-6 (probabilities <= 1)
  apply           fed with the GPU's own probabilities: the bf16 gate of the fused kernel (2e-2 abs, 1e-2 of max)
  composition     equals the fused forward within the same gate, and the oracle's attention forward
Guard elements after the score array and guard rows after sum_B must stay untouched.
"""
import numpy as np
import pytest
import torch

from oracle import unfused
from paper_2409_15373_amd.synthetic import make_custom, make_workload
from helpers import f64, gate_bf16, to_device

pytestmark = pytest.mark.gpu


def run_unfused(w, pad=5):
    from paper_2409_15373_amd import binding
    d = to_device(w, names=("q", "k", "v"), pad_rows=2)
    sq = binding.jfa_square_offsets(d["offsets"])
    sq_ref = unfused.square_offsets(w.offsets)
    assert sq.cpu().numpy().tolist() == sq_ref.tolist()
    S2 = int(sq_ref[-1])
    scores = torch.full((w.H * S2 + pad,), 777.0, dtype=torch.float32, device="cuda")
    binding.jfa_unfused_scores(d["q"], d["k"], d["offsets"], sq, w.max_len, scores)
    torch.cuda.synchronize()
    s_gpu = scores[:w.H * S2].reshape(w.H, S2).clone()
    binding.jfa_unfused_softmax(d["offsets"], sq, w.max_len, w.H, scores)
    torch.cuda.synchronize()
    p_gpu = scores[:w.H * S2].reshape(w.H, S2).clone()
    assert (scores[w.H * S2:] == 777.0).all(), "elements past the score array were written"
    out = torch.full_like(d["v"], 777.0)
    binding.jfa_unfused_apply(scores, d["v"], d["offsets"], sq, w.max_len, out=out)
    torch.cuda.synchronize()
    assert (out[w.sum_B:] == 777.0).all(), "guard rows of out were written"
    return s_gpu, p_gpu, out[:w.sum_B], d


@pytest.mark.parametrize("D,H,lengths", [
    (128, 2, [200, 1, 0, 77, 130, 33]),
    (64, 3, [5, 64, 129, 31]),
    (32, 1, [300, 2, 96]),
])
def test_unfused_steps_match_the_oracle(D, H, lengths):
    w = make_custom("unfused", lengths, H, D, "bf16", sigma=1.0, seed=11)
    s_gpu, p_gpu, out, _ = run_unfused(w)
    s_ref = unfused.scores(w.q, w.k, w.offsets)
    err = np.abs(f64(s_gpu) - s_ref) / np.maximum(1.0, np.abs(s_ref))
    assert err.max() <= 1e-4, f"scores: {err.max():.3e}"
    p_ref = unfused.softmax_rows(f64(s_gpu), w.offsets)             # softmax of the scores the GPU really had
    assert np.abs(f64(p_gpu) - p_ref).max() <= 2e-6
    o_ref = unfused.apply(f64(p_gpu), w.v, w.offsets)                # apply of the probabilities the GPU really had
    gate_bf16("apply", f64(out), o_ref)


def test_unfused_composition_matches_fused_forward_and_oracle(oracle):
    from paper_2409_15373_amd import binding
    w = make_custom("unfused", [257, 64, 1, 500, 0, 40], 2, 128, "bf16", sigma=1.0, seed=12)
    _, _, out_u, d = run_unfused(w)
    out_f, _ = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], 512)
    torch.cuda.synchronize()
    ref, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    gate_bf16("unfused vs oracle", f64(out_u), ref)
    gate_bf16("unfused vs fused", f64(out_u), f64(out_f[:w.sum_B]))


def test_unfused_on_the_geometric_workload(oracle):
    w = make_workload("c2_geom_bf16")
    _, _, out_u, _ = run_unfused(w)
    ref, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    gate_bf16("c2 unfused", f64(out_u), ref)


def test_unfused_full_size_on_sampled_blocks():
    """The benchmarked configuration: whole (sample, head) blocks picked from the 16 GB score array, each checked
    against the oracle run on that sample and head alone (longest, shortest and median sample, and random ones)."""
    from paper_2409_15373_amd import binding
    w = make_workload("c4_bimodal_bf16")
    d = to_device(w, names=("q", "k", "v"))
    sq = binding.jfa_square_offsets(d["offsets"])
    sq_ref = unfused.square_offsets(w.offsets)
    assert torch.equal(sq.cpu(), torch.from_numpy(sq_ref))
    S2 = int(sq_ref[-1])
    buf = torch.empty((w.H * S2,), dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(4)
    order = np.argsort(w.lengths)
    picks = [(int(order[-1]), 0), (int(order[0]), w.H - 1), (int(order[len(order) // 2]), 1)]
    picks += [(int(rng.integers(0, w.B)), int(rng.integers(0, w.H))) for _ in range(3)]

    def block(b, h):
        L = int(w.lengths[b])
        return f64(buf[h * S2 + int(sq_ref[b]): h * S2 + int(sq_ref[b + 1])]).reshape(1, L * L)

    def one(x, b, h):
        return np.ascontiguousarray(x[w.offsets[b]:w.offsets[b + 1], h:h + 1])

    binding.jfa_unfused_scores(d["q"], d["k"], d["offsets"], sq, w.max_len, buf)
    torch.cuda.synchronize()
    s_gpu = {}
    for b, h in picks:
        L = int(w.lengths[b])
        s_gpu[b, h] = block(b, h)
        s_ref = unfused.scores(one(w.q, b, h), one(w.k, b, h), np.array([0, L]))
        err = np.abs(s_gpu[b, h] - s_ref) / np.maximum(1.0, np.abs(s_ref))
        assert err.max() <= 1e-4, f"scores of sample {b} head {h}: {err.max():.3e}"
    binding.jfa_unfused_softmax(d["offsets"], sq, w.max_len, w.H, buf)
    out = binding.jfa_unfused_apply(buf, d["v"], d["offsets"], sq, w.max_len)
    torch.cuda.synchronize()
    for b, h in picks:
        L = int(w.lengths[b])
        p_gpu = block(b, h)
        p_ref = unfused.softmax_rows(s_gpu[b, h], np.array([0, L]))
        assert np.abs(p_gpu - p_ref).max() <= 2e-6, f"softmax of sample {b} head {h}"
        o_ref = unfused.apply(p_gpu, one(w.v, b, h), np.array([0, L]))
        gate_bf16(f"apply of sample {b} head {h}", f64(out[w.offsets[b]:w.offsets[b + 1], h:h + 1]), o_ref)


@pytest.mark.parametrize("D,H,lengths", [(128, 2, [200, 1, 0, 77, 130, 33]), (64, 2, [5, 64, 129, 300]), (32, 1, [70, 2])])
def test_unfused_backward_operators_match_the_oracle(D, H, lengths):
    """dP = product(dout, v, 1); dS = softmax_backward(P, dP, 1/sqrt(D)) in place; dV = apply_transposed(P, dout);
    dQ = apply(dS, k); dK = apply_transposed(dS, q): each against the oracle on the arrays the GPU really had."""
    from paper_2409_15373_amd import binding
    w = make_custom("unfused", lengths, H, D, "bf16", sigma=1.0, seed=13)
    d = to_device(w, names=("q", "k", "v", "dout"), pad_rows=2)
    sq = binding.jfa_square_offsets(d["offsets"])
    sq_ref = unfused.square_offsets(w.offsets); S2 = int(sq_ref[-1]); n = w.sum_B
    probs = torch.full((H * S2 + 5,), 777.0, dtype=torch.float32, device="cuda")
    binding.jfa_unfused_scores(d["q"], d["k"], d["offsets"], sq, w.max_len, probs)
    binding.jfa_unfused_softmax(d["offsets"], sq, w.max_len, H, probs)
    dp = torch.full((H * S2 + 5,), 555.0, dtype=torch.float32, device="cuda")
    binding.jfa_unfused_product(d["dout"], d["v"], d["offsets"], sq, w.max_len, 1.0, dp)
    torch.cuda.synchronize()
    P = f64(probs[:H * S2]).reshape(H, S2)
    dP = f64(dp[:H * S2]).reshape(H, S2)
    ref = unfused.product(w.dout, w.v, w.offsets, 1.0)
    assert (np.abs(dP - ref) / np.maximum(1.0, np.abs(ref))).max() <= 1e-4
    c = 1.0 / np.sqrt(D)
    binding.jfa_unfused_softmax_backward(probs, d["offsets"], sq, w.max_len, H, c, dp)
    torch.cuda.synchronize()
    assert (dp[H * S2:] == 555.0).all() and (probs[H * S2:] == 777.0).all(), "elements past the arrays were written"
    dS = f64(dp[:H * S2]).reshape(H, S2)
    ref = unfused.softmax_rows_backward(P, dP, w.offsets, c)
    assert np.abs(dS - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    outs = {}
    for name, arr, x in (("dv", probs, "dout"), ("dk", dp, "q")):
        o = torch.full_like(d["q"], 333.0)
        binding.jfa_unfused_apply_transposed(arr, d[x], d["offsets"], sq, w.max_len, out=o)
        torch.cuda.synchronize()
        assert (o[n:] == 333.0).all(), "guard rows were written"
        outs[name] = f64(o[:n])
    dq = binding.jfa_unfused_apply(dp, d["k"], d["offsets"], sq, w.max_len)
    torch.cuda.synchronize()
    gate_bf16("dV", outs["dv"], unfused.apply_transposed(P, w.dout, w.offsets), abs_tol=2e-2 * max(1.0, np.abs(outs["dv"]).max() / 4))
    gate_bf16("dK", outs["dk"], unfused.apply_transposed(dS, w.q, w.offsets))
    gate_bf16("dQ", f64(dq[:n]), unfused.apply(dS, w.k, w.offsets))


def test_unfused_backward_chain_matches_the_fused_backward(oracle):
    from paper_2409_15373_amd import binding
    w = make_custom("unfused", [257, 64, 1, 500, 0, 40], 2, 128, "bf16", sigma=1.0, seed=14)
    d = to_device(w, names=("q", "k", "v", "dout"))
    H, D = w.H, w.D
    sq = binding.jfa_square_offsets(d["offsets"])
    S2 = int(unfused.square_offsets(w.offsets)[-1])
    probs = torch.empty(H * S2, dtype=torch.float32, device="cuda"); dp = torch.empty_like(probs)
    binding.jfa_unfused_scores(d["q"], d["k"], d["offsets"], sq, 512, probs)
    binding.jfa_unfused_softmax(d["offsets"], sq, 512, H, probs)
    binding.jfa_unfused_product(d["dout"], d["v"], d["offsets"], sq, 512, 1.0, dp)
    dv = binding.jfa_unfused_apply_transposed(probs, d["dout"], d["offsets"], sq, 512)
    binding.jfa_unfused_softmax_backward(probs, d["offsets"], sq, 512, H, 1.0 / np.sqrt(D), dp)
    dq = binding.jfa_unfused_apply(dp, d["k"], d["offsets"], sq, 512)
    dk = binding.jfa_unfused_apply_transposed(dp, d["q"], d["offsets"], sq, 512)
    torch.cuda.synchronize()
    r_dq, r_dk, r_dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    for name, g, r in (("dq", dq, r_dq), ("dk", dk, r_dk), ("dv", dv, r_dv)):
        gate_bf16(name, f64(g), r, abs_tol=2e-2 * max(1.0, float(np.abs(r).max()) / 4))
