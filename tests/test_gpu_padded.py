"""The padded legs of the Figure 2 comparison (bench/figure2.py, bench/dense_compare.py) on tiny cases.

The paper's dense systems run on padded tensors (Section 3; Table 1's caption: the PyTorch versions need padding).
Two facts carry the comparison and are checked here against the oracle (bf16 gate: 2e-2 absolute, 1e-2 of the
tensor's maximum):

  1. the padded pipeline computes what the jagged kernels compute: pad q, k, v with jfa_jagged_to_dense, run
     attention on the padded tensor so that a sample's rows see that sample's valid keys only, unpad with
     jfa_dense_to_jagged -- the valid rows are the oracle's jagged attention (the oracle's own pin of this is its
     numpy padded-dense brute force).  Keys of the padding are masked through the offsets: the padded tensor of B
     samples is addressed as 2 B samples, sample b's L_b valid rows followed by its max_len - L_b padding rows
     (which attend among themselves and are dropped by the unpadding, as the padded query rows of a masked dense
     kernel are);
  2. the timed padded legs run the kernels with every sample max_len rows long (offsets 0, max_len, 2 max_len, ...):
     on such offsets the kernels are plain dense attention, compared here with the oracle on the same padded tensor.
"""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom, offsets_from_lengths
from helpers import f64, gate_bf16, to_device

pytestmark = pytest.mark.gpu
LENGTHS = [5, 130, 1, 64, 0, 77, 300]


@pytest.mark.parametrize("D,max_len", [(64, 300), (128, 300), (128, 320)])
@pytest.mark.parametrize("fused", [True, False])
def test_padded_pipeline_equals_jagged_attention_on_valid_rows(oracle, D, max_len, fused):
    from paper_2409_15373_amd import binding
    H = 2
    w = make_custom("padded", LENGTHS, H, D, dtype="bf16", seed=61, dout=False, max_len=max_len)
    d = to_device(w, names=("q", "k", "v"))
    B, off = w.B, d["offsets"]
    pad = lambda x: binding.jfa_jagged_to_dense(x, off, max_len, 0.0).view(B * max_len, H, D)
    qd, kd, vd = pad(d["q"]), pad(d["k"]), pad(d["v"])
    # the padded tensor as 2 B samples: valid rows of sample b, then its padding rows
    bounds = np.zeros(2 * B + 1, dtype=np.int64)
    bounds[1::2] = np.arange(B) * max_len + w.lengths
    bounds[2::2] = (np.arange(B) + 1) * max_len
    off2 = torch.from_numpy(bounds).cuda()
    if fused:
        out_d, lse_d = binding.jfa_forward(qd, kd, vd, off2, max_len)
    else:
        sq = binding.jfa_square_offsets(off2)
        pairs = int((np.diff(bounds) ** 2).sum())
        scores = torch.empty(H * pairs, dtype=torch.float32, device="cuda")
        binding.jfa_unfused_scores(qd, kd, off2, sq, max_len, scores)
        binding.jfa_unfused_softmax(off2, sq, max_len, H, scores)
        out_d = binding.jfa_unfused_apply(scores, vd, off2, sq, max_len)
    out = torch.full_like(d["q"], float("nan"))
    binding.jfa_dense_to_jagged(out_d.view(B, max_len, H, D), off, out)
    torch.cuda.synchronize()
    ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    gate_bf16("out", f64(out), ref_out)
    if fused:
        rows = np.concatenate([b * max_len + np.arange(L) for b, L in enumerate(w.lengths)])
        gate_bf16("lse", f64(lse_d)[:, rows], ref_lse)


def test_equal_length_offsets_are_dense_attention(oracle):
    """What the timed padded legs run: every sample max_len rows long."""
    from paper_2409_15373_amd import binding
    B, H, D, max_len = 3, 2, 128, 288
    w = make_custom("dense", [max_len] * B, H, D, dtype="bf16", seed=62, max_len=max_len)
    d = to_device(w)
    out, lse = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], max_len)
    dq, dk, dv, _ = binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], max_len)
    torch.cuda.synchronize()
    ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    rdq, rdk, rdv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    for name, got, ref in (("out", out, ref_out), ("lse", lse, ref_lse), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        gate_bf16(name, f64(got), ref)


def test_figure2_harness_runs_all_four_legs():
    from paper_2409_15373_amd.bench import figure2
    points = figure2.sweep(B=8, H=2, D=128, max_lens=[64, 320], reps=1)
    for p in points:
        for leg in ("dense", "jagged", "dense_flash", "jagged_flash"):
            assert p[leg]["fwd_us"] > 0 and p[leg]["bwd_us"] > 0 and p[leg]["fwd_bytes"] > 0
        assert p["dense"]["fwd_bytes"] > p["jagged"]["fwd_bytes"] > p["jagged_flash"]["fwd_bytes"]
        assert p["dense_flash"]["fwd_bytes"] > p["jagged_flash"]["fwd_bytes"]
