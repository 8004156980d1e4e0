"""bf16 MFMA backward vs the fp64 oracle on the same seeded bf16 inputs.

The backward consumes the GPU forward's own out and lse (as a training step would).  Gates as in the
forward test: per tensor, max |gpu - oracle| <= 2e-2 and max |gpu - oracle| / max |oracle| <= 1e-2.
"""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom, make_workload
from helpers import assert_guard_rows_untouched, f64, gate_bf16, sentinel_like, sentinel_stats, to_device

pytestmark = pytest.mark.gpu


def gpu_forward_backward(w, pad_rows=2, with_forward=False):
    """Outputs start as NaN in every valid row and as a guard pattern in the rows behind them."""
    from paper_2409_15373_amd import binding
    d = to_device(w, pad_rows=pad_rows)
    n = w.sum_B
    out = sentinel_like(d["q"], n)
    lse = sentinel_stats((w.H, n))
    binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], w.max_len, out=out, lse=lse)
    g = {x: sentinel_like(d["q"], n) for x in ("dq", "dk", "dv")}
    delta = sentinel_stats((2, w.H, n))   # plane 1: library scratch
    binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], w.max_len,
                         dq=g["dq"], dk=g["dk"], dv=g["dv"], delta=delta)
    torch.cuda.synchronize()
    for name, t in g.items():
        assert_guard_rows_untouched(name, t, n)
    if with_forward:
        return g["dq"][:n], g["dk"][:n], g["dv"][:n], delta[0], out[:n], lse
    return g["dq"][:n], g["dk"][:n], g["dv"][:n], delta[0]


@pytest.mark.parametrize("D", [32, 64, 128])
@pytest.mark.parametrize("H", [1, 3])
def test_bf16_backward_small_ragged(oracle, D, H):
    w = make_custom("ragged", [300, 1, 0, 129, 128, 127, 64, 33, 257, 2, 65, 0], H, D, dtype="bf16", seed=200 + D + H)
    dq, dk, dv, delta = gpu_forward_backward(w)
    rdq, rdk, rdv, rdelta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    gate_bf16("delta", f64(delta), rdelta, abs_tol=4e-2)       # |delta| reaches ~15: bf16 rounding of out dominates
    gate_bf16("dq", f64(dq), rdq)
    gate_bf16("dk", f64(dk), rdk)
    gate_bf16("dv", f64(dv), rdv)


def test_both_backward_paths_on_the_same_data(oracle):
    """D = 128: max_len <= 256 runs the dQ + fused dK/dV kernels, max_len > 256 the three direct-to-LDS kernels."""
    from paper_2409_15373_amd import binding
    w = make_custom("both", [256, 130, 1, 77, 0, 200, 33], 2, 128, dtype="bf16", seed=21)
    rdq, rdk, rdv, rdelta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    d = to_device(w)
    for max_len in (256, 257):
        out, lse = binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], max_len)
        dq, dk, dv, delta = binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], max_len)
        torch.cuda.synchronize()
        gate_bf16(f"dq(max_len={max_len})", f64(dq), rdq)
        gate_bf16(f"dk(max_len={max_len})", f64(dk), rdk)
        gate_bf16(f"dv(max_len={max_len})", f64(dv), rdv)


def test_bf16_backward_length_one(oracle):
    w = make_custom("ones", [1] * 21, 2, 64, dtype="bf16", seed=7)
    dq, dk, dv, _ = gpu_forward_backward(w)
    np.testing.assert_array_equal(f64(dv), w.dout.astype(np.float64))          # P = 1 exactly
    assert np.abs(f64(dq)).max() <= 1e-2 and np.abs(f64(dk)).max() <= 1e-2     # dS = P (dP - delta) ~ 0


@pytest.mark.parametrize("name", ["c5_uniform_bf16", "c4_bimodal_bf16"])
def test_full_size_backward_on_sampled_pairs(oracle, name):
    """The configuration with gradients and the benchmarked one, as the benchmark runs them (same inputs, same launch
    shapes); whole (sample, head) pairs -- longest, shortest, median and random ones -- against the oracle."""
    w = make_workload(name, with_dout=True)
    dq, dk, dv, delta = gpu_forward_backward(w)
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    order = np.argsort(w.lengths)
    rng = np.random.default_rng(2)
    pairs = {(int(order[-1]), 0), (int(order[0]), w.H - 1), (int(order[len(order) // 2]), 1)}
    while len(pairs) < 16:
        pairs.add((int(rng.integers(0, w.B)), int(rng.integers(0, w.H))))
    pairs = sorted(pairs)
    rdq, rdk, rdv, rdelta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets, pairs=pairs)
    rows = np.concatenate([np.arange(w.offsets[b], w.offsets[b + 1]) for b, _ in pairs])
    heads = np.concatenate([np.full(int(w.lengths[b]), h) for b, h in pairs])
    gate_bf16("dq", f64(dq)[rows, heads], rdq[rows, heads])
    gate_bf16("dk", f64(dk)[rows, heads], rdk[rows, heads])
    gate_bf16("dv", f64(dv)[rows, heads], rdv[rows, heads])
    gate_bf16("delta", f64(delta)[heads, rows], rdelta[heads, rows], abs_tol=4e-2)


def test_backward_is_deterministic():
    w = make_custom("det", [700, 90, 1, 333], 2, 128, dtype="bf16", seed=3)
    a = gpu_forward_backward(w)
    b = gpu_forward_backward(w)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("is_causal", [False, True])
def test_many_short_samples_with_dynamic_claims(oracle, is_causal):
    """The direct-to-LDS kernels on a batch of 1300 short samples (some empty) and three long ones: several work items per
    workgroup, so that items are claimed dynamically (one atomic per item on the die's queue) and, with more than 1024
    samples, decoded from the schedule in global memory by the wave-wide 64-ary search."""
    from oracle import causal
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(31)
    lengths = rng.integers(0, 49, size=1300)
    lengths[[7, 650, 1299]] = [300, 520, 257]
    w = make_custom("many", lengths, 2, 128, dtype="bf16", seed=32, max_len=600)
    d = to_device(w, pad_rows=2)
    n = w.sum_B
    out = sentinel_like(d["q"], n)
    lse = sentinel_stats((w.H, n))
    binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], 600, out=out, lse=lse, causal=is_causal)
    g = {x: sentinel_like(d["q"], n) for x in ("dq", "dk", "dv")}
    delta = sentinel_stats((2, w.H, n))
    binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], 600,
                         dq=g["dq"], dk=g["dk"], dv=g["dv"], delta=delta, causal=is_causal)
    torch.cuda.synchronize()
    assert (out[n:] == 777.0).all() and all((t[n:] == 777.0).all() for t in g.values()), "guard rows were written"
    if is_causal:
        r_out, r_lse = causal.forward(w.q, w.k, w.v, w.offsets)
        rdq, rdk, rdv, _ = causal.backward(w.q, w.k, w.v, w.dout, w.offsets)
    else:
        r_out, r_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
        rdq, rdk, rdv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    # gradients of short, peaked samples reach several units: the absolute gate follows the tensor's scale (bf16 rounding
    # of a value x alone is |x| / 512), the relative gate is unchanged
    scaled = lambda r: 2e-2 * max(1.0, float(np.abs(r).max()) / 2)
    gate_bf16("out", f64(out[:n]), r_out)
    gate_bf16("lse", f64(lse), r_lse)
    gate_bf16("dq", f64(g["dq"][:n]), rdq, abs_tol=scaled(rdq))
    gate_bf16("dk", f64(g["dk"][:n]), rdk, abs_tol=scaled(rdk))
    gate_bf16("dv", f64(g["dv"][:n]), rdv, abs_tol=scaled(rdv))
