"""jfa_forward_noalloc, the forward entry point that allocates nothing (its work table is a fixed array in device
memory), called through the C ABI: two calls in a row on one stream, the second with a smaller batch, each compared
with jfa_forward on the same inputs.  Both run the same kernels on the same schedule, so the results must be equal
bit for bit; they are also checked against the oracle to the bf16 gate (max |gpu - oracle| <= 2e-2 and <= 1e-2 of
the tensor's maximum).  Collected last: a failure here must not hide the other GPU tests.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom
from helpers import f64, gate_bf16, to_device

pytestmark = pytest.mark.gpu


def raw_forward(fn, d, B, max_len, H, D, out, lse):
    """The C entry point itself: device pointers and sizes, torch's current stream."""
    vp = ctypes.c_void_p
    st = fn(vp(d["q"].data_ptr()), vp(d["k"].data_ptr()), vp(d["v"].data_ptr()), vp(d["offsets"].data_ptr()),
            ctypes.c_int64(B), ctypes.c_int64(max_len), ctypes.c_int(H), ctypes.c_int(D), vp(out.data_ptr()),
            vp(lse.data_ptr()), vp(torch.cuda.current_stream().cuda_stream))
    return st


def case(rng_seed, B, hi, H, D, max_len):
    rng = np.random.default_rng(rng_seed)
    lengths = rng.integers(0, hi + 1, size=B)
    lengths[0] = hi
    return make_custom("noalloc", lengths, H, D, dtype="bf16", seed=rng_seed, dout=False, max_len=max_len)


def test_two_calls_in_a_row_match_jfa_forward(oracle):
    from paper_2409_15373_amd import binding
    lib = binding.load()
    cases = [case(71, 900, 700, 2, 128, 1024),      # direct-to-LDS kernel, several work items per workgroup
             case(72, 9, 300, 2, 128, 1024),        # the same kernel on a much smaller batch: stale table contents behind it
             case(73, 40, 200, 3, 64, 256)]         # register-staged kernel
    for w in cases:
        d = to_device(w, names=("q", "k", "v"))
        n = w.sum_B
        nan = float("nan")
        out_a = torch.full_like(d["q"], nan); lse_a = torch.full((w.H, n), nan, dtype=torch.float32, device="cuda")
        out_b = torch.full_like(d["q"], nan); lse_b = torch.full((w.H, n), nan, dtype=torch.float32, device="cuda")
        assert raw_forward(lib.jfa_forward_noalloc, d, w.B, w.max_len, w.H, w.D, out_a, lse_a) == 0, lib.jfa_last_error()
        assert raw_forward(lib.jfa_forward, d, w.B, w.max_len, w.H, w.D, out_b, lse_b) == 0, lib.jfa_last_error()
        torch.cuda.synchronize()
        assert torch.isfinite(out_a.float()).all() and torch.isfinite(lse_a).all(), "rows that were never written"
        assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b), f"B = {w.B}: results differ from jfa_forward"
        ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets)
        gate_bf16("out", f64(out_a), ref_out)
        gate_bf16("lse", f64(lse_a), ref_lse)


def test_batches_beyond_the_fixed_table_are_refused():
    from paper_2409_15373_amd import binding
    lib = binding.load()
    w = case(74, 3, 40, 1, 64, 64)
    d = to_device(w, names=("q", "k", "v"))
    out = torch.full_like(d["q"], 5.0); lse = torch.zeros((w.H, w.sum_B), dtype=torch.float32, device="cuda")
    st = raw_forward(lib.jfa_forward_noalloc, d, 65537, w.max_len, w.H, w.D, out, lse)
    torch.cuda.synchronize()
    assert st == binding.JFA_ERR_UNSUPPORTED and b"JFA_NOALLOC_MAX_B" in lib.jfa_last_error()
    assert (out == 5.0).all(), "a refused call must not launch anything"
