"""Table 1's jagged feature operators on the GPU vs oracle/feature_ops.py on the same seeded bf16 inputs.

Outputs are bf16 roundings of fp32 accumulations of bf16 products: the gate is the bf16 gate of the attention
tests, max |gpu - oracle| <= 1e-2 * max |oracle| (and 2e-2 absolute, scaled up with the output's magnitude where
sums over hundreds of rows exceed 1).  Guard rows after sum_B must stay untouched.
"""
import numpy as np
import pytest
import torch

from oracle import feature_ops as fo
from paper_2409_15373_amd.synthetic import offsets_from_lengths, round_to_bf16_bits, bf16_bits_to_f32, lengths_for
from helpers import f64, gate_bf16

pytestmark = pytest.mark.gpu

LENGTHS = [300, 1, 0, 129, 128, 127, 64, 33, 257, 2, 65, 0]
GUARD = 2


def bf16_pair(rng, shape, sigma=1.0):
    """(float32 array holding exact bf16 values, the same as a CUDA bf16 tensor)."""
    bits = round_to_bf16_bits((rng.standard_normal(shape) * sigma).astype(np.float32))
    return bf16_bits_to_f32(bits), torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def guarded(t, value=777.0):
    """t with GUARD extra rows of `value` appended; returns (whole buffer, view of the first rows)."""
    buf = torch.cat([t, torch.full((GUARD,) + tuple(t.shape[1:]), value, dtype=t.dtype, device=t.device)])
    return buf, buf[:t.shape[0]]


def scaled_gate(name, got, ref):
    gate_bf16(name, got, ref, abs_tol=2e-2 * max(1.0, float(np.abs(ref).max())))


@pytest.mark.parametrize("D,T", [(64, 64), (128, 128), (32, 128), (128, 32), (64, 32), (32, 32)])
def test_bmm_pair_matches_the_oracle(D, T):
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(D * 7 + T)
    off = offsets_from_lengths(np.array(LENGTHS)); n = int(off[-1]); B = len(LENGTHS)
    offd = torch.from_numpy(off).cuda()
    x, xd = bf16_pair(rng, (n, D)); y, yd = bf16_pair(rng, (n, T)); w, wd = bf16_pair(rng, (B, D, T), 0.5)
    xbuf, _ = guarded(xd, float("nan")); ybuf, _ = guarded(yd, float("nan"))
    obuf = torch.full((n + GUARD, T), 777.0, dtype=torch.bfloat16, device="cuda")
    binding.jfa_jagged_dense_bmm(xbuf, wd, offd, 512, out=obuf)
    torch.cuda.synchronize()
    assert (obuf[n:] == 777.0).all(), "guard rows of out were written"
    scaled_gate("jagged_dense_bmm", f64(obuf[:n]), fo.jagged_dense_bmm(x, w, off))
    got = binding.jfa_jagged_jagged_bmm(xbuf, ybuf, offd, 512)
    torch.cuda.synchronize()
    ref = fo.jagged_jagged_bmm(x, y, off)
    scaled_gate("jagged_jagged_bmm", f64(got), ref)
    assert (f64(got)[[2, 11]] == 0).all(), "empty samples give zero blocks"


@pytest.mark.parametrize("D", [32, 64, 128])
def test_softmax_and_backward_match_the_oracle(D):
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(D)
    off = offsets_from_lengths(np.array(LENGTHS)); n = int(off[-1])
    offd = torch.from_numpy(off).cuda()
    x, xd = bf16_pair(rng, (n, D), 2.0)
    xbuf, _ = guarded(xd, float("nan"))
    ybuf = torch.full((n + GUARD, D), 777.0, dtype=torch.bfloat16, device="cuda")
    binding.jfa_jagged_softmax(xbuf, offd, 512, y=ybuf)
    torch.cuda.synchronize()
    assert (ybuf[n:] == 777.0).all()
    y_ref = fo.jagged_softmax(x, off)
    gate_bf16("jagged_softmax", f64(ybuf[:n]), y_ref)
    # backward on the probabilities the GPU really produced (bf16) and a bf16 dy
    dy, dyd = bf16_pair(rng, (n, D))
    dybuf, _ = guarded(dyd, float("nan"))
    dxbuf = torch.full((n + GUARD, D), 555.0, dtype=torch.bfloat16, device="cuda")
    ybuf[n:] = float("nan")
    binding.jfa_jagged_softmax_backward(ybuf, dybuf, offd, 512, dx=dxbuf)
    torch.cuda.synchronize()
    assert (dxbuf[n:] == 555.0).all()
    gate_bf16("jagged_softmax_backward", f64(dxbuf[:n]), fo.jagged_softmax_backward(f64(ybuf[:n]), dy, off))


def test_softmax_large_values_and_long_sample():
    """Columns with values around +-80 (exp overflows without the running maximum) and one sample of 5000 rows."""
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(3)
    off = offsets_from_lengths(np.array([5000, 3, 40])); n = int(off[-1])
    x, xd = bf16_pair(rng, (n, 64), 30.0)
    y = binding.jfa_jagged_softmax(xd, torch.from_numpy(off).cuda(), 5000)
    torch.cuda.synchronize()
    assert np.isfinite(f64(y)).all()
    gate_bf16("jagged_softmax", f64(y), fo.jagged_softmax(x, off))


def test_feature_ops_on_a_table_sized_workload():
    """B = 1024 samples with lengths uniform on [1, 200], D = T = 64: every sample of jagged_jagged_bmm and sampled
    rows of the others against the oracle."""
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(11)
    L = lengths_for("uniform", 1024, 200, np.random.Generator(np.random.PCG64(5)))
    off = offsets_from_lengths(L); n = int(off[-1]); offd = torch.from_numpy(off).cuda()
    x, xd = bf16_pair(rng, (n, 64)); y, yd = bf16_pair(rng, (n, 64)); w, wd = bf16_pair(rng, (1024, 64, 64), 0.5)
    scaled_gate("jagged_dense_bmm", f64(binding.jfa_jagged_dense_bmm(xd, wd, offd, 200)), fo.jagged_dense_bmm(x, w, off))
    scaled_gate("jagged_jagged_bmm", f64(binding.jfa_jagged_jagged_bmm(xd, yd, offd, 200)), fo.jagged_jagged_bmm(x, y, off))
    gate_bf16("jagged_softmax", f64(binding.jfa_jagged_softmax(xd, offd, 200)), fo.jagged_softmax(x, off))
