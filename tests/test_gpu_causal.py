"""Causal jagged self attention on the GPU vs oracle/causal.py, forward and backward, fp32 and bf16.

Gates as for the non-causal path (fp32 2e-5 relative to max(1, |ref|); bf16 2e-2 absolute and 1e-2 of the tensor's
maximum).  Lengths cover several row tiles and 64-key stages, tiles whose diagonal crosses stage boundaries, ragged
tails, and samples of length 0 and 1; D = 128 runs with max_len <= 256 (register-staged kernels) and with
max_len > 256 (direct-to-LDS kernels: 256-row tiles, the masking stages around the diagonal, the stream of dK / dV
starting at the tile's first key).
"""
import numpy as np
import pytest
import torch

from oracle import causal
from paper_2409_15373_amd.synthetic import make_custom
from helpers import f64, gate_bf16, gate_f32, to_device

pytestmark = pytest.mark.gpu
GUARD = 2


def run(w, max_len):
    from paper_2409_15373_amd import binding
    d = to_device(w, names=("q", "k", "v", "dout"), pad_rows=GUARD)
    n, H = w.sum_B, w.H
    out = torch.full_like(d["q"], 777.0)
    lse = torch.full((H, n), 777.0, dtype=torch.float32, device="cuda")
    binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], max_len, out=out, lse=lse, causal=True)
    torch.cuda.synchronize()
    assert (out[n:] == 777.0).all()
    grads = [torch.full_like(d["q"], 555.0) for _ in range(3)]
    stats = torch.empty((2 if w.dtype == "bf16" else 1, H, n), dtype=torch.float32, device="cuda")
    out_in = out.clone(); out_in[n:] = float("nan")
    binding.jfa_backward(d["q"], d["k"], d["v"], out_in, d["dout"], lse, d["offsets"], max_len, dq=grads[0], dk=grads[1],
                         dv=grads[2], delta=stats, causal=True)
    torch.cuda.synchronize()
    for g in grads:
        assert (g[n:] == 555.0).all(), "guard rows of a gradient were written"
    got = dict(out=f64(out[:n]), lse=f64(lse), dq=f64(grads[0][:n]), dk=f64(grads[1][:n]), dv=f64(grads[2][:n]), delta=f64(stats[0]))
    r_out, r_lse = causal.forward(w.q, w.k, w.v, w.offsets)
    r_dq, r_dk, r_dv, r_delta = causal.backward(w.q, w.k, w.v, w.dout, w.offsets)
    ref = dict(out=r_out, lse=r_lse, dq=r_dq, dk=r_dk, dv=r_dv, delta=r_delta)
    for name in got:
        if w.dtype == "f32":
            gate_f32(name, got[name], ref[name], tol=2e-5, relative_to_one=True)
        else:
            gate_bf16(name, got[name], ref[name], abs_tol=2e-2 * max(1.0, float(np.abs(ref[name]).max()) / 4))


LENGTHS = [300, 1, 0, 129, 128, 127, 64, 33, 257, 2, 65, 0, 200]


@pytest.mark.parametrize("D", [32, 128])
def test_causal_fp32(D):
    run(make_custom("causal", [70, 1, 0, 64, 65, 130], 2, D, dtype="f32", seed=21 + D), 130)


@pytest.mark.parametrize("D,H", [(32, 1), (64, 3), (128, 2)])
def test_causal_bf16(D, H):
    run(make_custom("causal", LENGTHS, H, D, dtype="bf16", seed=22 + D), 512 if D != 128 else 256)


@pytest.mark.parametrize("lengths", [[1000, 513, 64, 700, 1], [256, 257, 0, 255, 300, 65, 2, 1281, 768]])
def test_causal_bf16_long_samples(lengths):
    run(make_custom("causal", lengths, 2, 128, dtype="bf16", seed=23), 2048)


def test_causal_first_row_returns_v_and_later_rows_ignore_the_future():
    """Exact properties: row 0 of every sample returns its value row (p = 1); changing rows after i leaves row i as it was."""
    from paper_2409_15373_amd import binding
    w = make_custom("causal", [150, 40], 2, 64, dtype="bf16", seed=24, dout=False)
    d = to_device(w, names=("q", "k", "v"))
    out, lse = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], 256, causal=True)
    k2, v2 = d["k"].clone(), d["v"].clone()
    k2[100:150] = 3.0; v2[100:150] = -7.0                      # the future of rows 0 .. 99 of sample 0
    out2, lse2 = binding.jfa_forward(d["q"], k2, v2, d["offsets"], 256, causal=True)
    torch.cuda.synchronize()
    for s in (0, 150):
        assert torch.equal(out[s].view(torch.int16), d["v"][s].view(torch.int16))
    assert torch.equal(out[:100].view(torch.int16), out2[:100].view(torch.int16)) and torch.equal(lse[:, :100], lse2[:, :100])
    assert not torch.equal(out[100:150].view(torch.int16), out2[100:150].view(torch.int16))


def test_causal_stale_reference_maximum_takes_the_conservative_pass():
    """Direct-to-LDS forward: the first 40 keys score 0 and the later ones ~724, so the fixed reference maximum (first
    32 keys) is far too low for every query past row 40: the tile is redone maximum-first, with the causal mask."""
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.synthetic import round_to_bf16_bits
    lengths = [300, 500, 40]
    w = make_custom("stale", lengths, 1, 128, dtype="bf16", seed=12, dout=False, max_len=512)
    q = np.full_like(w.q, 8.0)
    k = np.zeros_like(w.k)
    for b, L in enumerate(lengths):
        s0 = int(w.offsets[b])
        k[s0 + 40: s0 + L] = 8.0
    w.q, w.k = q, k
    w.bits["q"], w.bits["k"] = round_to_bf16_bits(q), round_to_bf16_bits(k)
    d = to_device(w, names=("q", "k", "v"))
    out, lse = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], 512, causal=True)
    torch.cuda.synchronize()
    r_out, r_lse = causal.forward(w.q, w.k, w.v, w.offsets)
    assert np.isfinite(f64(out)).all() and np.isfinite(f64(lse)).all()
    gate_bf16("out", f64(out), r_out)
    gate_bf16("lse", f64(lse), r_lse, abs_tol=2e-2 * max(1.0, np.abs(r_lse).max() / 4))


def test_causal_full_size_on_sampled_pairs():
    """The benchmarked configuration's inputs through the causal entry points (what variants_bench times); whole
    (sample, head) pairs -- longest, shortest, median and random ones -- against the oracle run on each pair alone."""
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.synthetic import make_workload
    w = make_workload("c4_bimodal_bf16", with_dout=True)
    d = to_device(w)
    nan_like = lambda t: torch.full_like(t, float("nan"))   # every row has to be written: an unwritten tile stays NaN
    out, lse = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], w.max_len, causal=True, out=nan_like(d["q"]),
                                   lse=torch.full((w.H, w.sum_B), float("nan"), dtype=torch.float32, device="cuda"))
    dq, dk, dv, _ = binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], w.max_len, causal=True,
                                         dq=nan_like(d["q"]), dk=nan_like(d["q"]), dv=nan_like(d["q"]))
    torch.cuda.synchronize()
    for name, t in (("out", out), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
        assert torch.isfinite(t.float()).all(), f"{name}: rows that were never written (or not finite)"
    order = np.argsort(w.lengths)
    rng = np.random.default_rng(6)
    picks = [(int(order[-1]), 0), (int(order[0]), w.H - 1), (int(order[len(order) // 2]), 1)]
    picks += [(int(rng.integers(0, w.B)), int(rng.integers(0, w.H))) for _ in range(5)]
    for b, h in picks:
        s, e = int(w.offsets[b]), int(w.offsets[b + 1])
        one = lambda x: np.ascontiguousarray(x[s:e, h:h + 1])
        off1 = np.array([0, e - s], dtype=np.int64)
        r_out, r_lse = causal.forward(one(w.q), one(w.k), one(w.v), off1)
        r_dq, r_dk, r_dv, _ = causal.backward(one(w.q), one(w.k), one(w.v), one(w.dout), off1)
        tag = f"sample {b} (length {e - s}) head {h}: "
        gate_bf16(tag + "out", f64(out[s:e, h:h + 1]), r_out)
        gate_bf16(tag + "lse", f64(lse[h:h + 1, s:e]), r_lse)
        for name, g, r in (("dq", dq, r_dq), ("dk", dk, r_dk), ("dv", dv, r_dv)):
            gate_bf16(tag + name, f64(g[s:e, h:h + 1]), r, abs_tol=2e-2 * max(1.0, float(np.abs(r).max()) / 2))
