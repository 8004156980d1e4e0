"""Seeded random shapes: many small configurations of lengths, heads and head sizes through every attention entry
point (self, cross, causal; register-staged and direct-to-LDS kernels), forward and backward against the oracles.

Each case draws B in [1, 12], H in [1, 4], D from {32, 64, 128} and lengths from a mix of 0, 1, tile and stage
boundaries +- 1 and arbitrary values up to 700, so ragged tails, empty samples and boundary lengths meet in
combinations no hand-written case lists.  Gates as in the other bf16 tests.
"""
import numpy as np
import pytest
import torch

from oracle import causal as causal_oracle, cross as cross_oracle
from paper_2409_15373_amd.synthetic import offsets_from_lengths, round_to_bf16_bits, bf16_bits_to_f32
from helpers import f64, gate_bf16

pytestmark = pytest.mark.gpu
SPECIAL = [0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513]


def draw_lengths(rng, B, cap):
    L = np.where(rng.random(B) < 0.5, rng.choice(SPECIAL, B), rng.integers(0, 701, B))
    return np.minimum(L, cap)


def bf16_tensor(rng, n, H, D, sigma):
    bits = round_to_bf16_bits((rng.standard_normal((n, H, D)) * sigma).astype(np.float32))
    return bf16_bits_to_f32(bits), torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def scaled(name, got, ref):
    """The bf16 gate with its absolute part following the tensor's scale once that exceeds 2 (gradients that sum
    hundreds of rows): then the relative part, 1e-2 of the maximum, is the one that binds."""
    gate_bf16(name, got, ref, abs_tol=2e-2 * max(1.0, float(np.abs(ref).max()) / 2))


def self_case(seed):
    rng = np.random.default_rng(1000 + seed)
    B, H, D = int(rng.integers(1, 13)), int(rng.integers(1, 5)), int(rng.choice([32, 64, 128]))
    cap = 256 if seed % 2 else 700                      # max_len <= 256 keeps D = 128 on the register-staged kernels
    L = draw_lengths(rng, B, cap)
    off = offsets_from_lengths(L); n = int(off[-1])
    if n == 0:
        L[0] = 5; off = offsets_from_lengths(L); n = int(off[-1])
    tensors = [bf16_tensor(rng, n, H, D, 1.0) for _ in range(4)]
    return B, H, D, cap, L, off, n, tensors


# Seeds of a one-off sweep over seeds 12 .. 331 (640 self / causal runs, 320 cross runs) that end outside the relative
# gate against the exact oracle: (seed, causal, tensor, measured max error / max |oracle|).  In both, a sample of two
# rows holds the tensor's largest error: dS = P o (dP - delta) is a small difference of large numbers there (|delta|
# 6 .. 14) and delta is formed, as the interface defines it, from the bf16 forward output: in fp64 arithmetic with that
# one substitution (oracle/given_out.py) the gradients are already 1.1 % and 1.3 .. 1.7 % of the maximum away.
KNOWN_OUTSIDE = [(165, False, "dq", 1.17e-2), (324, True, "dk", 1.35e-2)]


@pytest.mark.parametrize("seed,is_causal,tensor,measured", KNOWN_OUTSIDE)
def test_known_cases_outside_the_gate_are_inherited_from_the_bf16_output(oracle, seed, is_causal, tensor, measured):
    """Against the backward evaluated in fp64 from the SAME bf16 forward output (what any implementation of the
    interface is given) the standard gate holds; against the exact oracle the error stays below twice the gate."""
    from oracle import given_out
    from paper_2409_15373_amd import binding
    B, H, D, cap, L, off, n, ((q, qd), (k, kd), (v, vd), (do, dod)) = self_case(seed)
    offd = torch.from_numpy(off).cuda()
    lse = torch.empty((H, n), dtype=torch.float32, device="cuda")
    stats = torch.empty((2, H, n), dtype=torch.float32, device="cuda")
    out, _ = binding.jfa_forward(qd, kd, vd, offd, cap, lse=lse, causal=is_causal)
    dq, dk, dv, _ = binding.jfa_backward(qd, kd, vd, out, dod, lse, offd, cap, delta=stats, causal=is_causal)
    torch.cuda.synchronize()
    g_dq, g_dk, g_dv, _ = given_out.backward(q, k, v, f64(out), do, off, causal=is_causal)
    scaled("dq vs fp64 from the same out", f64(dq), g_dq)
    scaled("dk vs fp64 from the same out", f64(dk), g_dk)
    scaled("dv vs fp64 from the same out", f64(dv), g_dv)
    exact = causal_oracle.backward(q, k, v, do, off) if is_causal else oracle.backward(q, k, v, do, off)
    for name, got, ref in (("dq", dq, exact[0]), ("dk", dk, exact[1]), ("dv", dv, exact[2])):
        gate_bf16(name + " vs the exact oracle", f64(got), ref, abs_tol=2e-2 * max(1.0, float(np.abs(ref).max()) / 2), rel_tol=2e-2)


@pytest.mark.parametrize("seed", range(12))
def test_random_self_and_causal(oracle, seed):
    from paper_2409_15373_amd import binding
    B, H, D, cap, L, off, n, ((q, qd), (k, kd), (v, vd), (do, dod)) = self_case(seed)
    offd = torch.from_numpy(off).cuda()
    for is_causal in (False, True):
        lse = torch.empty((H, n), dtype=torch.float32, device="cuda")
        stats = torch.empty((2, H, n), dtype=torch.float32, device="cuda")
        out, _ = binding.jfa_forward(qd, kd, vd, offd, cap, lse=lse, causal=is_causal)
        dq, dk, dv, _ = binding.jfa_backward(qd, kd, vd, out, dod, lse, offd, cap, delta=stats, causal=is_causal)
        torch.cuda.synchronize()
        if is_causal:
            r_out, r_lse = causal_oracle.forward(q, k, v, off)
            r_dq, r_dk, r_dv, _ = causal_oracle.backward(q, k, v, do, off)
        else:
            r_out, r_lse = oracle.forward(q, k, v, off)
            r_dq, r_dk, r_dv, _ = oracle.backward(q, k, v, do, off)
        tag = f"seed {seed} B {B} H {H} D {D} causal {is_causal} L {L.tolist()}: "
        scaled(tag + "out", f64(out), r_out); scaled(tag + "lse", f64(lse), r_lse)
        scaled(tag + "dq", f64(dq), r_dq); scaled(tag + "dk", f64(dk), r_dk); scaled(tag + "dv", f64(dv), r_dv)


@pytest.mark.parametrize("seed", range(8))
def test_random_cross(seed):
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(2000 + seed)
    B, H, D = int(rng.integers(1, 13)), int(rng.integers(1, 5)), int(rng.choice([32, 64, 128]))
    cap = 256 if seed % 2 else 700
    Lq, Lk = draw_lengths(rng, B, cap), draw_lengths(rng, B, cap)
    Lq[0] = max(Lq[0], 3); Lk[0] = max(Lk[0], 3)          # at least one sample with both sides
    oq, ok = offsets_from_lengths(Lq), offsets_from_lengths(Lk)
    nq, nk = int(oq[-1]), int(ok[-1])
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    (q, qd), (do, dod) = (bf16_tensor(rng, nq, H, D, 1.0) for _ in range(2))
    (k, kd), (v, vd) = (bf16_tensor(rng, nk, H, D, 1.0) for _ in range(2))
    lse = torch.empty((H, nq), dtype=torch.float32, device="cuda")
    stats = torch.empty((2, H, nq), dtype=torch.float32, device="cuda")
    out, _ = binding.jfa_forward_cross(qd, kd, vd, oqd, okd, cap, cap, lse=lse)
    dq, dk, dv, _ = binding.jfa_backward_cross(qd, kd, vd, out, dod, lse, oqd, okd, cap, cap, delta=stats)
    torch.cuda.synchronize()
    r_out, r_lse = cross_oracle.forward(q, k, v, oq, ok)
    r_dq, r_dk, r_dv, _ = cross_oracle.backward(q, k, v, do, oq, ok)
    fin = np.isfinite(r_lse[0])
    tag = f"seed {seed} B {B} H {H} D {D} Lq {Lq.tolist()} Lk {Lk.tolist()}: "
    assert np.isneginf(f64(lse)[:, ~fin]).all()
    scaled(tag + "out", f64(out), r_out); scaled(tag + "lse", f64(lse)[:, fin], r_lse[:, fin])
    scaled(tag + "dq", f64(dq), r_dq); scaled(tag + "dk", f64(dk), r_dk); scaled(tag + "dv", f64(dv), r_dv)


@pytest.mark.parametrize("seed", range(8))
def test_random_cross_with_few_queries(seed):
    """At most 32 queries per sample at D = 128 (the few-query kernels): B up to 400 so that some draws take the
    schedule and tickets (more than four items per workgroup) and others the static deal; key lists of 0 .. 700 rows
    with the boundary lengths mixed in."""
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(3000 + seed)
    B, H, D = int(rng.choice([1, 3, 40, 400])), int(rng.integers(1, 5)), 128
    Lq = np.where(rng.random(B) < 0.3, rng.choice([0, 1, 31, 32], B), rng.integers(0, 33, B))
    Lk = draw_lengths(rng, B, 700)
    Lq[0] = max(Lq[0], 3); Lk[0] = max(Lk[0], 3)
    oq, ok = offsets_from_lengths(Lq), offsets_from_lengths(Lk)
    nq, nk = int(oq[-1]), int(ok[-1])
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    (q, qd), (do, dod) = (bf16_tensor(rng, nq, H, D, 1.0) for _ in range(2))
    (k, kd), (v, vd) = (bf16_tensor(rng, nk, H, D, 1.0) for _ in range(2))
    nan = float("nan")   # rows of samples that have both queries and keys must all be written
    lse = torch.full((H, nq), nan, dtype=torch.float32, device="cuda")
    out = torch.full((nq, H, D), nan, dtype=torch.bfloat16, device="cuda")
    stats = torch.empty((2, H, nq), dtype=torch.float32, device="cuda")
    dq = torch.full((nq, H, D), nan, dtype=torch.bfloat16, device="cuda")
    dk, dv = (torch.full((nk, H, D), nan, dtype=torch.bfloat16, device="cuda") for _ in range(2))
    binding.jfa_forward_cross(qd, kd, vd, oqd, okd, 32, 700, out=out, lse=lse)
    binding.jfa_backward_cross(qd, kd, vd, out, dod, lse, oqd, okd, 32, 700, dq=dq, dk=dk, dv=dv, delta=stats)
    torch.cuda.synchronize()
    r_out, r_lse = cross_oracle.forward(q, k, v, oq, ok)
    r_dq, r_dk, r_dv, _ = cross_oracle.backward(q, k, v, do, oq, ok)
    fin = np.isfinite(r_lse[0])
    tag = f"seed {seed} B {B} H {H}: "
    assert np.isneginf(f64(lse)[:, ~fin]).all()
    scaled(tag + "out", f64(out), r_out); scaled(tag + "lse", f64(lse)[:, fin], r_lse[:, fin])
    scaled(tag + "dq", f64(dq), r_dq); scaled(tag + "dk", f64(dk), r_dk); scaled(tag + "dv", f64(dv), r_dv)
