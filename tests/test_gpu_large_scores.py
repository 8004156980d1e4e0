"""Large random scores through the direct-to-LDS kernels (D = 128, samples longer than 256 rows), forward and backward,
self, causal and cross attention.

Queries and keys are drawn with standard deviation 2 and 4, so scaled scores q.k / sqrt(D) have standard deviation 4
and 16 and reach +-15 and +-70: an error of relative size e in a score changes its probability by |score| * e, which is
what shows any rounding applied to the operands of the score product (the kernels keep q and k exact and apply
log2(e) / sqrt(D) in fp32 on the accumulator, as Section 2.1's softmax(Q K^T / sqrt(D)) of the given bf16 values
requires).  Values and dout stay at standard deviation 1, so out is gated with the plain bf16 gate (2e-2 absolute and
1e-2 of the tensor's maximum); lse and the gradients exceed a few units, where bf16 / fp32 rounding of a value x alone
costs |x| / 512, so their absolute gate follows the tensor's scale and the relative gate of 1e-2 binds.
"""
import numpy as np
import pytest
import torch

from oracle import causal as causal_oracle, cross as cross_oracle
from paper_2409_15373_amd.synthetic import offsets_from_lengths, round_to_bf16_bits, bf16_bits_to_f32
from helpers import f64, gate_bf16

pytestmark = pytest.mark.gpu
H, D = 2, 128
LQ = [600, 300, 257, 1000, 40, 1]
LK = [520, 300, 700, 64, 290, 333]


def bf16_pair(rng, n, sigma):
    bits = round_to_bf16_bits((rng.standard_normal((n, H, D)) * sigma).astype(np.float32))
    return bf16_bits_to_f32(bits), torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def scaled(name, got, ref):
    return gate_bf16(name, got, ref, abs_tol=2e-2 * max(1.0, float(np.abs(ref).max()) / 2))


def nan_buffers(nq, nk):
    nan = float("nan")
    mk = lambda n: torch.full((n, H, D), nan, dtype=torch.bfloat16, device="cuda")
    return mk(nq), torch.full((H, nq), nan, dtype=torch.float32, device="cuda"), mk(nq), mk(nk), mk(nk)


@pytest.mark.parametrize("sigma", [2.0, 4.0])
@pytest.mark.parametrize("mode", ["self", "causal", "cross"])
def test_large_scores_on_the_direct_to_lds_kernels(oracle, mode, sigma):
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(int(sigma) * 10 + len(mode))
    oq = offsets_from_lengths(np.array(LQ))
    ok = offsets_from_lengths(np.array(LK)) if mode == "cross" else oq
    nq, nk = int(oq[-1]), int(ok[-1])
    (q, qd), (do, dod) = bf16_pair(rng, nq, sigma), bf16_pair(rng, nq, 1.0)
    (k, kd), (v, vd) = bf16_pair(rng, nk, sigma), bf16_pair(rng, nk, 1.0)
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    out, lse, dq, dk, dv = nan_buffers(nq, nk)
    stats = torch.empty((2, H, nq), dtype=torch.float32, device="cuda")
    max_len = 1024                                          # > 256 at D = 128: the direct-to-LDS kernels
    if mode == "cross":
        binding.jfa_forward_cross(qd, kd, vd, oqd, okd, max_len, max_len, out=out, lse=lse)
        binding.jfa_backward_cross(qd, kd, vd, out, dod, lse, oqd, okd, max_len, max_len, dq=dq, dk=dk, dv=dv, delta=stats)
        r_out, r_lse = cross_oracle.forward(q, k, v, oq, ok)
        r_dq, r_dk, r_dv, _ = cross_oracle.backward(q, k, v, do, oq, ok)
    else:
        is_causal = mode == "causal"
        binding.jfa_forward(qd, kd, vd, oqd, max_len, out=out, lse=lse, causal=is_causal)
        binding.jfa_backward(qd, kd, vd, out, dod, lse, oqd, max_len, dq=dq, dk=dk, dv=dv, delta=stats, causal=is_causal)
        if is_causal:
            r_out, r_lse = causal_oracle.forward(q, k, v, oq)
            r_dq, r_dk, r_dv, _ = causal_oracle.backward(q, k, v, do, oq)
        else:
            r_out, r_lse = oracle.forward(q, k, v, oq)
            r_dq, r_dk, r_dv, _ = oracle.backward(q, k, v, do, oq)
    torch.cuda.synchronize()
    tag = f"{mode} sigma {sigma}: "
    res = [gate_bf16(tag + "out", f64(out), r_out), scaled(tag + "lse", f64(lse), r_lse),
           scaled(tag + "dq", f64(dq), r_dq), scaled(tag + "dk", f64(dk), r_dk), scaled(tag + "dv", f64(dv), r_dv)]
    print(tag + "  ".join(f"{n} {a:.2e}/{r:.2e}" for n, (a, r) in zip(("out", "lse", "dq", "dk", "dv"), res)), flush=True)
