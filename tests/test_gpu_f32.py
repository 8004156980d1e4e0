"""fp32 HIP path vs the fp64 oracle: max abs error 1e-5 on out and gradients, 1e-5 relative-to-max(1,|x|) on lse."""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom, make_workload
from helpers import f64, gate_f32, to_device

pytestmark = pytest.mark.gpu


def run_case(oracle, w, pad_rows=3):
    from paper_2409_15373_amd import binding
    d = to_device(w, pad_rows=pad_rows)
    n = w.sum_B
    out = torch.full_like(d["q"], 777.0)
    lse = torch.full((w.H, n), 777.0, dtype=torch.float32, device="cuda")
    # lse of a padded buffer: the kernel addresses lse as [H, sum_B] with sum_B = offsets[B]
    binding.jfa_forward(d["q"], d["k"], d["v"], d["offsets"], w.max_len, out=out, lse=lse)
    torch.cuda.synchronize()
    ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
    gate_f32("out", f64(out[:n]), ref_out)
    gate_f32("lse", f64(lse), ref_lse, relative_to_one=True)
    assert (out[n:] == 777.0).all(), "guard rows of out were written"
    if w.dout is not None:
        dq = torch.full_like(d["q"], 777.0); dk = torch.full_like(d["q"], 777.0); dv = torch.full_like(d["q"], 777.0)
        delta = torch.full((w.H, n), 777.0, dtype=torch.float32, device="cuda")
        binding.jfa_backward(d["q"], d["k"], d["v"], out, d["dout"], lse, d["offsets"], w.max_len, dq=dq, dk=dk, dv=dv, delta=delta)
        torch.cuda.synchronize()
        rdq, rdk, rdv, rdelta = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
        gate_f32("delta", f64(delta), rdelta, tol=2e-5)
        # gradients sum up to L_b products of O(1) terms: scale the fp32 tolerance with the magnitude
        gate_f32("dq", f64(dq[:n]), rdq, tol=2e-5, relative_to_one=True)
        gate_f32("dk", f64(dk[:n]), rdk, tol=2e-5, relative_to_one=True)
        gate_f32("dv", f64(dv[:n]), rdv, tol=2e-5, relative_to_one=True)
        for g in (dq, dk, dv):
            assert (g[n:] == 777.0).all(), "guard rows of a gradient were written"


def test_config1_tiny_fp32(oracle):
    w = make_workload("c1_tiny_f32")
    assert w.lengths.tolist() == [55, 41, 33, 18]
    run_case(oracle, w)


@pytest.mark.parametrize("D", [32, 64, 128])
def test_fp32_ragged_multi_tile(oracle, D):
    # spans several 64-row tiles, ragged tails, zero-length and length-1 samples
    w = make_custom("ragged", [130, 0, 1, 64, 65, 7, 0, 200], 2, D, dtype="f32", seed=D)
    run_case(oracle, w)


def test_fp32_empty_batch_and_all_empty_samples(oracle):
    from paper_2409_15373_amd import binding
    e = torch.empty((0, 2, 32), dtype=torch.float32, device="cuda")
    off = torch.zeros(1, dtype=torch.int64, device="cuda")
    out, lse = binding.jfa_forward(e, e, e, off, 0)            # B = 0
    off = torch.zeros(4, dtype=torch.int64, device="cuda")
    g = torch.zeros((4, 2, 32), dtype=torch.float32, device="cuda")   # non-null pointers, B = 3 empty samples
    out = torch.full_like(g, 5.0); lse = torch.full((2, 4), 5.0, dtype=torch.float32, device="cuda")
    binding.jfa_forward(g, g, g, off, 16, out=out, lse=lse)
    torch.cuda.synchronize()
    assert (out == 5.0).all() and (lse == 5.0).all()
