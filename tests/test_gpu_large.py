"""Tensors beyond 2^31 elements (and 4 GB): every row offset in the kernels has to be 64-bit.

B = 12 samples of up to 4096 rows with H = 512 heads of D = 128: [sum_B, H, D] bf16 tensors of about 5 GB each,
rows 128 KB apart.  Inputs are drawn on the device; a few (sample, head) pairs, among them the last sample's last
head (the highest addresses), are copied to the host and checked against the oracle run on that pair alone.
The forward and backward of the benchmarked path (direct-to-LDS kernels) are exercised: one launch each.
"""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import offsets_from_lengths
from helpers import f64, gate_bf16

pytestmark = pytest.mark.gpu


def _one(t, s, e, h):
    """[L, 1, D] float32 host copy of rows s .. e - 1, head h."""
    return t[s:e, h:h + 1].float().cpu().numpy()


def test_tensors_over_4_gb(oracle):
    from paper_2409_15373_amd import binding
    H, D = 512, 128
    L = np.array([4096, 3000, 4095, 1, 0, 4096, 2049, 4000, 4096, 4096, 4096, 4096])
    off = offsets_from_lengths(L); n = int(off[-1])
    assert n * H * D > 2**31
    gen = torch.Generator(device="cuda").manual_seed(5)
    mk = lambda s: (torch.randn(n, H, D, device="cuda", generator=gen, dtype=torch.bfloat16) * s)
    q, k, v, dout = mk(0.5), mk(0.5), mk(1.0), mk(1.0)
    offd = torch.from_numpy(off).cuda()
    out, lse = binding.jfa_forward(q, k, v, offd, 4096)
    dq, dk, dv, delta = binding.jfa_backward(q, k, v, out, dout, lse, offd, 4096)
    torch.cuda.synchronize()
    for b, h in [(11, H - 1), (0, 0), (3, 17), (6, 300), (11, 0)]:
        s, e = int(off[b]), int(off[b + 1])
        one_off = np.array([0, e - s])
        qs, ks, vs, ds = (_one(t, s, e, h) for t in (q, k, v, dout))
        r_out, r_lse = oracle.forward(qs, ks, vs, one_off)
        gate_bf16(f"out[{b},{h}]", f64(out[s:e, h:h + 1]), r_out)
        gate_bf16(f"lse[{b},{h}]", f64(lse[h:h + 1, s:e]), r_lse)
        r_dq, r_dk, r_dv, r_delta = oracle.backward(qs, ks, vs, ds, one_off)
        for name, g, r in (("dq", dq, r_dq), ("dk", dk, r_dk), ("dv", dv, r_dv)):
            gate_bf16(f"{name}[{b},{h}]", f64(g[s:e, h:h + 1]), r, abs_tol=2e-2 * max(1.0, float(np.abs(r).max()) / 4))
        gate_bf16(f"delta[{b},{h}]", f64(delta[h:h + 1, s:e]), r_delta, abs_tol=2e-2 * max(1.0, float(np.abs(r_delta).max()) / 4))
