"""The autograd wrappers are marshalling only: their outputs and gradients are the entry points' own, bit for bit, and
(on a small case) match the fp64 oracle within the stated gate."""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_custom, offsets_from_lengths
from helpers import f64, gate_bf16, to_device

pytestmark = pytest.mark.gpu


def _rand(n, H, D, dtype, gen):
    return torch.randn(n, H, D, device="cuda", generator=gen).to(dtype)


@pytest.mark.parametrize("dtype,causal,L", [(torch.bfloat16, False, [300, 5, 0, 64, 700]), (torch.bfloat16, True, [300, 5, 0, 64, 700]),
                                            (torch.float32, False, [40, 3, 0, 17])])
def test_self_attention_wrapper_equals_the_entry_points(dtype, causal, L):
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.autograd import jagged_flash_attention
    H, D = 2, 128 if dtype == torch.bfloat16 else 32
    off = torch.from_numpy(offsets_from_lengths(np.array(L))).cuda()
    n, max_len = int(off[-1]), max(L)
    gen = torch.Generator(device="cuda").manual_seed(1)
    q, k, v, dout = (_rand(n, H, D, dtype, gen) for _ in range(4))
    qa, ka, va = (t.clone().requires_grad_(True) for t in (q, k, v))
    out = jagged_flash_attention(qa, ka, va, off, max_len, causal=causal)
    out.backward(dout)
    r_out, r_lse = binding.jfa_forward(q, k, v, off, max_len, causal=causal)
    r_dq, r_dk, r_dv, _ = binding.jfa_backward(q, k, v, r_out, dout, r_lse, off, max_len, causal=causal)
    torch.cuda.synchronize()
    for name, a, b in (("out", out, r_out), ("dq", qa.grad, r_dq), ("dk", ka.grad, r_dk), ("dv", va.grad, r_dv)):
        assert torch.equal(a.detach().view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if dtype == torch.bfloat16 else torch.int32)), name


@pytest.mark.parametrize("max_q", [32, 200])
def test_cross_attention_wrapper_equals_the_entry_points(max_q):
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.autograd import jagged_flash_cross_attention
    rng = np.random.default_rng(2)
    B, H, D = 12, 2, 128
    Lq, Lk = rng.integers(0, max_q + 1, B), rng.integers(0, 600, B)
    oq, ok = (torch.from_numpy(offsets_from_lengths(x)).cuda() for x in (Lq, Lk))
    nq, nk = int(oq[-1]), int(ok[-1])
    gen = torch.Generator(device="cuda").manual_seed(3)
    q, dout = _rand(nq, H, D, torch.bfloat16, gen), _rand(nq, H, D, torch.bfloat16, gen)
    k, v = _rand(nk, H, D, torch.bfloat16, gen), _rand(nk, H, D, torch.bfloat16, gen)
    qa, ka, va = (t.clone().requires_grad_(True) for t in (q, k, v))
    out = jagged_flash_cross_attention(qa, ka, va, oq, ok, max_q, 599)
    out.backward(dout)
    r_out, r_lse = binding.jfa_forward_cross(q, k, v, oq, ok, max_q, 599)
    r_dq, r_dk, r_dv, _ = binding.jfa_backward_cross(q, k, v, r_out, dout, r_lse, oq, ok, max_q, 599)
    torch.cuda.synchronize()
    for name, a, b in (("out", out, r_out), ("dq", qa.grad, r_dq), ("dk", ka.grad, r_dk), ("dv", va.grad, r_dv)):
        assert torch.equal(a.detach().view(torch.int16), b.view(torch.int16)), name


def test_gradients_through_the_wrapper_match_the_oracle():
    """A scalar loss sum(out * w) differentiated by torch through the wrapper against the oracle's gradients for dout = w."""
    import oracle
    from paper_2409_15373_amd.autograd import jagged_flash_attention
    w = make_custom("autograd", [70, 1, 33, 130, 300], H=2, D=128, dtype="bf16", seed=11, dout=True)
    d = to_device(w)
    qa, ka, va = (d[n].clone().requires_grad_(True) for n in ("q", "k", "v"))
    out = jagged_flash_attention(qa, ka, va, d["offsets"], w.max_len)
    (out.float() * d["dout"].float()).sum().backward()
    torch.cuda.synchronize()
    r_out, _ = oracle.forward(w.q, w.k, w.v, w.offsets)
    r_dq, r_dk, r_dv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets)
    gate_bf16("out", f64(out), r_out)
    gate_bf16("dq", f64(qa.grad), r_dq)
    gate_bf16("dk", f64(ka.grad), r_dk)
    gate_bf16("dv", f64(va.grad), r_dv)
