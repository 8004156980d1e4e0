"""Whole-tensor checks of the full-size configurations, in the launch shapes the benchmark times.

Sampled (sample, head) pairs (tests/test_gpu_bf16_fwd.py, _bwd.py) cannot show a work item that is dropped or decoded
to the wrong place outside the sample, so every element is covered here:
  * every output buffer starts as NaN in its valid rows: a tile that is never written fails the isfinite check;
  * c3, c4, c5 (forward) and c5 (backward, the configuration with gradients) are compared with the oracle element by
    element over the whole tensor (the backward is cut into parts so that no single test is silent for long);
  * delta is compared over the whole tensor with rowsum(dout * out) of the tensors the call was given;
  * every configuration's backward gets identities that hold per (sample, head) at any size and are evaluated on the
    GPU over the whole tensor (Section 2.1's softmax is a convex weighting, Section 2.2's gradients inherit
    sum_j dS_ij = 0):
        out[i, :] lies in the per-feature hull of the sample's V rows,
        sum_j dK_j = 0,   sum_j dV_j = sum_i dO_i,
    with tolerances derived from the bf16 rounding of L_b terms (see the functions).
Gate of the element-wise comparisons: max |gpu - oracle| <= 2e-2 and max |gpu - oracle| / max |oracle| <= 1e-2 per
tensor; `delta` against the oracle: within the bf16 rounding of the `out` it is computed from, row by row.
"""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_workload
from helpers import f64, gate_bf16
from test_gpu_bf16_bwd import gpu_forward_backward

pytestmark = pytest.mark.gpu
_cache = {}


def results(name):
    """Forward + backward of a named configuration on the GPU, computed once per test session."""
    if name not in _cache:
        _cache.clear()                       # one configuration resident at a time
        w = make_workload(name, with_dout=True)
        dq, dk, dv, delta, out, lse = gpu_forward_backward(w, with_forward=True)
        for label, t in (("out", out), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv), ("delta", delta)):
            assert torch.isfinite(t.float()).all(), f"{name}: {label} has rows that were never written (or not finite)"
        # a6, whole tensor: delta is rowsum(dO o O) of the tensors the call was given, accumulated in fp32
        dd = (_bits_to_device(w, "dout").double() * out.double()).sum(dim=2).T           # [H, sum_B]
        err = (delta.double() - dd).abs().max().item()
        assert err <= 1e-4, f"{name}: delta differs from rowsum(dout * out) of its own inputs by {err:.2e}"
        _cache[name] = (w, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv, delta=delta))
    return _cache[name]


def _bits_to_device(w, name):
    return torch.from_numpy(w.bits[name].view(np.int16)).view(torch.bfloat16).cuda()


def segment_sum(x, w):
    """[sum_B, H, D] -> [B, H, D] fp32 sums over each sample's rows."""
    seg = torch.repeat_interleave(torch.arange(w.B, device="cuda"), torch.from_numpy(w.lengths).cuda())
    return torch.zeros((w.B,) + tuple(x.shape[1:]), dtype=torch.float32, device="cuda").index_add_(0, seg, x.float())


def segment_extreme(x, w, how):
    seg = torch.repeat_interleave(torch.arange(w.B, device="cuda"), torch.from_numpy(w.lengths).cuda())
    init = float("inf") if how == "amin" else float("-inf")
    idx = seg[:, None, None].expand(-1, x.shape[1], x.shape[2])
    return torch.full((w.B,) + tuple(x.shape[1:]), init, dtype=torch.float32, device="cuda").scatter_reduce_(
        0, idx, x.float(), how, include_self=True)


@pytest.mark.parametrize("name", ["c3_zipf_bf16", "c4_bimodal_bf16", "c5_uniform_bf16"])
def test_whole_tensor_identities(name):
    w, g = results(name)
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    seg = torch.repeat_interleave(torch.arange(w.B, device="cuda"), torch.from_numpy(w.lengths).cuda())
    L = torch.from_numpy(w.lengths).cuda().float()[:, None, None]
    # out is a convex combination of the sample's V rows: inside their hull up to the bf16 rounding of out (2^-9
    # relative) and of the probabilities (2^-9 relative each, so at most 2^-8 of the largest |v| in total)
    v = dev(w.bits["v"])
    lo, hi = segment_extreme(v, w, "amin"), segment_extreme(v, w, "amax")
    slack = 2.0 ** -7 * torch.maximum(lo.abs(), hi.abs()) + 1e-6
    out = g["out"].float()
    below = (lo - slack)[seg] - out
    above = out - (hi + slack)[seg]
    assert below.max().item() <= 0 and above.max().item() <= 0, f"{name}: out leaves the hull of its sample's V rows"
    # sum_j dK_j = 0: exact for exact dS (rows of dS sum to zero); here dS and dK are rounded to bf16, independent
    # roundings of L_b terms of size <= max|dK| / 512, so the sum stays below a few sqrt(L_b) roundings
    dk_sum = segment_sum(g["dk"], w)
    dk_max = segment_extreme(g["dk"].abs(), w, "amax").amax(dim=2, keepdim=True)
    bound = 0.02 * torch.sqrt(L) * torch.clamp(dk_max, min=1.0)
    ratio = (dk_sum.abs() / bound).max().item()
    assert ratio <= 1.0, f"{name}: sum_j dK_j is {ratio:.2f} x its rounding bound"
    # sum_j dV_j = sum_i dO_i (columns of P^T sum the rows of P, which sum to one up to the bf16 rounding of P)
    dv_sum = segment_sum(g["dv"], w)
    do_sum = segment_sum(dev(w.bits["dout"]), w)
    dv_max = segment_extreme(g["dv"].abs(), w, "amax").amax(dim=2, keepdim=True)
    bound = 0.02 * torch.sqrt(L) * torch.clamp(dv_max, min=1.0)
    ratio_v = ((dv_sum - do_sum).abs() / bound).max().item()
    assert ratio_v <= 1.0, f"{name}: sum_j dV_j - sum_i dO_i is {ratio_v:.2f} x its rounding bound"
    print(f"{name}: identities hold; sum dK at {ratio:.3f} and sum dV - sum dO at {ratio_v:.3f} of their bounds", flush=True)


@pytest.mark.parametrize("name", ["c3_zipf_bf16", "c4_bimodal_bf16", "c5_uniform_bf16"])
def test_forward_whole_tensor_against_the_oracle(oracle, name):
    w, g = results(name)
    ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    a = gate_bf16("out", f64(g["out"]), ref_out)
    b = gate_bf16("lse", f64(g["lse"]), ref_lse)
    print(f"{name}: out max abs {a[0]:.2e} rel {a[1]:.2e}; lse max abs {b[0]:.2e} rel {b[1]:.2e}", flush=True)


N_PARTS = 4


@pytest.mark.parametrize("part", range(N_PARTS))
def test_c5_backward_whole_tensor_against_the_oracle(oracle, part):
    """All (sample, head) pairs of c5 whose sample index is congruent to `part` mod N_PARTS."""
    w, g = results("c5_uniform_bf16")
    pairs = [(b, h) for b in range(part, w.B, N_PARTS) for h in range(w.H)]
    rdq, rdk, rdv, rdelta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets, pairs=pairs)
    rows = np.concatenate([np.arange(w.offsets[b], w.offsets[b + 1]) for b in range(part, w.B, N_PARTS)])
    for label, ref in (("dq", rdq), ("dk", rdk), ("dv", rdv)):
        assert np.isfinite(ref[rows]).all()
        a = gate_bf16(label, f64(g[label][rows]), ref[rows])
        print(f"c5 part {part}: {label} max abs {a[0]:.2e} rel {a[1]:.2e}", flush=True)
    # delta = rowsum(dO o O) is taken from the bf16 forward output the call is given: against the oracle's (exact O) it
    # may differ, row by row, by the rounding of O to bf16 (2^-9 relative per element) plus as much again for the
    # kernel's own error in O before rounding
    dout, out = f64(_bits_to_device(w, "dout")[rows]), f64(g["out"][rows])
    bound = 2.0 ** -8 * np.abs(dout * out).sum(axis=2).T + 1e-3                     # [H, rows]
    excess = np.abs(f64(g["delta"][:, rows]) - rdelta[:, rows]) / bound
    assert excess.max() <= 1.0, f"delta differs from the oracle by {excess.max():.2f} x the rounding bound of its row"
