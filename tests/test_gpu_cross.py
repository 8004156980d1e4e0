"""Jagged cross attention (separate query and key offsets) on the GPU vs oracle/cross.py, forward and backward.

Gates as for self attention: fp32 1e-5 (relative to max(1, |ref|)), bf16 2e-2 absolute and 1e-2 of the tensor's
maximum.  Samples without keys must give out = 0, lse = -inf, dq = 0; samples without queries dk = dv = 0; guard rows
after the last query and key rows must stay untouched.  Through the cross entry points with equal offsets the
results must equal the self-attention entry points bit for bit (same arithmetic, other template instance).
"""
import numpy as np
import pytest
import torch

from oracle import cross
from paper_2409_15373_amd.synthetic import offsets_from_lengths, round_to_bf16_bits, bf16_bits_to_f32
from helpers import f64, gate_bf16, gate_f32

pytestmark = pytest.mark.gpu
GUARD = 2


def make(Lq, Lk, H, D, dtype, seed, sigma=1.0):
    """Host arrays (float32 holding the exact values) and guarded device tensors for q, k, v, dout."""
    rng = np.random.default_rng(seed)
    oq, ok = offsets_from_lengths(np.array(Lq)), offsets_from_lengths(np.array(Lk))
    host, dev = {}, {}
    for name, n, s in (("q", oq[-1], sigma), ("k", ok[-1], sigma), ("v", ok[-1], 1.0), ("dout", oq[-1], 1.0)):
        x = (rng.standard_normal((int(n), H, D)) * s).astype(np.float32)
        if dtype == "bf16":
            bits = round_to_bf16_bits(x)
            x = bf16_bits_to_f32(bits)
            t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
        else:
            t = torch.from_numpy(x)
        host[name] = x
        dev[name] = torch.cat([t, torch.full((GUARD, H, D), float("nan"), dtype=t.dtype)]).cuda()   # rows past the end: never read
    return host, dev, oq, ok


def run(Lq, Lk, H, D, dtype, seed, max_len_q, max_len_kv, sigma=1.0):
    from paper_2409_15373_amd import binding
    host, dev, oq, ok = make(Lq, Lk, H, D, dtype, seed, sigma)
    nq, nk = int(oq[-1]), int(ok[-1])
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    tdt = dev["q"].dtype
    out = torch.full((nq + GUARD, H, D), 777.0, dtype=tdt, device="cuda")
    lse = torch.full((H, nq), 777.0, dtype=torch.float32, device="cuda")
    binding.jfa_forward_cross(dev["q"], dev["k"], dev["v"], oqd, okd, max_len_q, max_len_kv, out=out, lse=lse)
    torch.cuda.synchronize()
    assert (out[nq:] == 777.0).all(), "guard rows of out were written"
    dq = torch.full((nq + GUARD, H, D), 555.0, dtype=tdt, device="cuda")
    dk = torch.full((nk + GUARD, H, D), 555.0, dtype=tdt, device="cuda")
    dv = torch.full((nk + GUARD, H, D), 555.0, dtype=tdt, device="cuda")
    out_in = out.clone(); out_in[nq:] = float("nan")
    stats = torch.empty((2 if dtype == "bf16" else 1, H, nq), dtype=torch.float32, device="cuda")   # sized by the real row count
    binding.jfa_backward_cross(dev["q"], dev["k"], dev["v"], out_in, dev["dout"], lse, oqd, okd, max_len_q, max_len_kv,
                               dq=dq, dk=dk, dv=dv, delta=stats)
    torch.cuda.synchronize()
    delta = stats[0]
    assert (dq[nq:] == 555.0).all() and (dk[nk:] == 555.0).all() and (dv[nk:] == 555.0).all(), "guard rows of a gradient were written"
    got = dict(out=f64(out[:nq]), lse=f64(lse), dq=f64(dq[:nq]), dk=f64(dk[:nk]), dv=f64(dv[:nk]), delta=f64(delta))
    r_out, r_lse = cross.forward(host["q"], host["k"], host["v"], oq, ok)
    # the backward consumed the GPU's own out and lse: the oracle's gradients are those of the exact forward
    r_dq, r_dk, r_dv, r_delta = cross.backward(host["q"], host["k"], host["v"], host["dout"], oq, ok)
    ref = dict(out=r_out, lse=r_lse, dq=r_dq, dk=r_dk, dv=r_dv, delta=r_delta)
    return got, ref, oq, ok


def compare(got, ref, dtype, oq, ok, Lq, Lk):
    empty_q_rows = np.concatenate([np.arange(oq[b], oq[b + 1]) for b in range(len(Lq)) if Lk[b] == 0] + [np.array([], dtype=np.int64)]).astype(np.int64)
    fin = np.ones(ref["lse"].shape[1], dtype=bool); fin[empty_q_rows] = False
    assert np.isneginf(got["lse"][:, ~fin]).all() and np.isneginf(ref["lse"][:, ~fin]).all()
    assert (got["out"][~fin] == 0).all() and (got["dq"][~fin] == 0).all()
    for b in range(len(Lq)):
        if Lq[b] == 0:
            assert (got["dk"][ok[b]:ok[b + 1]] == 0).all() and (got["dv"][ok[b]:ok[b + 1]] == 0).all()
    pairs = [("out", got["out"], ref["out"]), ("lse", got["lse"][:, fin], ref["lse"][:, fin]), ("dq", got["dq"], ref["dq"]),
             ("dk", got["dk"], ref["dk"]), ("dv", got["dv"], ref["dv"]), ("delta", got["delta"][:, fin], ref["delta"][:, fin])]
    for name, g, r in pairs:
        if dtype == "f32":
            gate_f32(name, g, r, tol=2e-5, relative_to_one=True)
        else:
            gate_bf16(name, g, r, abs_tol=2e-2 * max(1.0, float(np.abs(r).max()) / 4))


LQ = [37, 1, 0, 70, 64, 5, 130]
LK = [5, 90, 12, 0, 64, 129, 1]


@pytest.mark.parametrize("D", [32, 128])
def test_cross_fp32(D):
    got, ref, oq, ok = run(LQ, LK, 2, D, "f32", 1, 130, 129)
    compare(got, ref, "f32", oq, ok, LQ, LK)


@pytest.mark.parametrize("D,H", [(32, 1), (64, 3), (128, 2)])
def test_cross_bf16_register_staged_kernels(D, H):
    Lq = [300, 1, 0, 129, 128, 33, 65, 200]
    Lk = [40, 257, 12, 0, 128, 300, 1, 64]
    got, ref, oq, ok = run(Lq, Lk, H, D, "bf16", 2, 256, 256)      # max_len <= 256 keeps D = 128 on these kernels too
    compare(got, ref, "bf16", oq, ok, Lq, Lk)


def test_cross_bf16_direct_to_lds_kernels():
    Lq = [300, 1, 0, 129, 700, 33, 257, 64]
    Lk = [513, 64, 40, 0, 65, 1000, 31, 1]
    got, ref, oq, ok = run(Lq, Lk, 2, 128, "bf16", 3, 1024, 1024)   # D = 128 and max_len > 256: the long-sample kernels
    compare(got, ref, "bf16", oq, ok, Lq, Lk)


@pytest.mark.parametrize("Lq,Lk", [
    ([1, 32, 0, 5, 32, 17, 8, 3], [513, 64, 40, 0, 65, 1000, 31, 1]),     # every kind of block: full, ragged, one key; no queries; no keys
    ([8] * 40, [300 + 7 * i for i in range(40)]),                          # ragged last blocks of every residue
    ([32, 1], [2100, 4096]),                                               # many blocks per wave: both buffers in turn, partial sums of all four waves
    ([5] * 12, [1, 31, 32, 33, 64, 96, 127, 128, 129, 160, 161, 256]),     # fewer blocks than waves, as many, one more
])
def test_cross_few_queries_backward_in_one_pass(Lq, Lk):
    """At most 32 queries per sample at D = 128: the backward is one kernel that reads K and V once (dQ from the sum of
    the waves' partial blocks, dK and dV complete per block of keys)."""
    got, ref, oq, ok = run(Lq, Lk, 2, 128, "bf16", 5, 32, max(Lk))
    compare(got, ref, "bf16", oq, ok, Lq, Lk)


def test_cross_few_queries_many_items_per_workgroup():
    """3600 (sample, head) items for at most 256 workgroups: every workgroup runs a dozen items one after the other,
    with samples without queries and without keys among them (the LDS tiles, the copy buffers and the partial sums
    of one item are reused by the next)."""
    rng = np.random.default_rng(3)
    B = 900
    Lq, Lk = rng.integers(0, 33, B), rng.integers(0, 200, B)
    got, ref, oq, ok = run(Lq, Lk, 4, 128, "bf16", 6, 32, 199)
    compare(got, ref, "bf16", oq, ok, Lq, Lk)


@pytest.mark.parametrize("max_len", [256, 1024])
def test_cross_with_equal_offsets_is_self_attention(max_len):
    """Bit for bit wherever both entry points run the same kernels."""
    from paper_2409_15373_amd import binding
    L = [300, 1, 0, 129, 64, 700 if max_len > 256 else 250]
    host, dev, oq, _ = make(L, L, 2, 128, "bf16", 4)
    od = torch.from_numpy(oq).cuda()
    n = int(oq[-1])
    lse_s, lse_x = (torch.empty((2, n), dtype=torch.float32, device="cuda") for _ in range(2))   # sized by the real row count
    out_s, _ = binding.jfa_forward(dev["q"], dev["k"], dev["v"], od, max_len, lse=lse_s)
    out_x, _ = binding.jfa_forward_cross(dev["q"], dev["k"], dev["v"], od, od.clone(), max_len, max_len, lse=lse_x)
    torch.cuda.synchronize()
    assert torch.equal(out_s[:n].view(torch.int16), out_x[:n].view(torch.int16)) and torch.equal(lse_s, lse_x)
    st_s, st_x = (torch.empty((2, 2, n), dtype=torch.float32, device="cuda") for _ in range(2))
    gs = binding.jfa_backward(dev["q"], dev["k"], dev["v"], out_s, dev["dout"], lse_s, od, max_len, delta=st_s)
    gx = binding.jfa_backward_cross(dev["q"], dev["k"], dev["v"], out_s, dev["dout"], lse_s, od, od.clone(), max_len, max_len, delta=st_x)
    torch.cuda.synchronize()
    for name, a, b in zip(("dq", "dk", "dv"), gs[:3], gx[:3]):
        if max_len > 256 and name != "dq":
            # long samples: self attention computes dK and dV in one kernel, in which dS is formed from the bf16
            # probabilities that dV uses; the cross entry point runs them as two kernels with fp32 probabilities in
            # dS.  Both are within rounding of each other, no longer the same bits.
            diff = (a[:n].float() - b[:n].float()).abs().max().item()
            assert diff <= 2.0 ** -7 * max(1.0, a[:n].float().abs().max().item()), (name, diff)
        else:
            assert torch.equal(a[:n].view(torch.int16), b[:n].view(torch.int16)), name


def test_cross_stale_reference_maximum_takes_the_conservative_pass():
    """Direct-to-LDS forward with separate lengths: the first 40 keys of a sample score 0 and the later ones ~724, far
    above the fixed reference maximum of the first 32 keys: the tile is redone maximum-first."""
    from paper_2409_15373_amd import binding
    Lq, Lk = [300, 70, 10], [500, 300, 40]
    host, dev, oq, ok = make(Lq, Lk, 1, 128, "bf16", 9)
    q = np.full_like(host["q"], 8.0)
    k = np.zeros_like(host["k"])
    for b in range(3):
        k[ok[b] + 40: ok[b + 1]] = 8.0
    guard = torch.full((GUARD, 1, 128), float("nan"), dtype=torch.bfloat16)
    qd = torch.cat([torch.from_numpy(round_to_bf16_bits(q).view(np.int16)).view(torch.bfloat16), guard]).cuda()
    kd = torch.cat([torch.from_numpy(round_to_bf16_bits(k).view(np.int16)).view(torch.bfloat16), guard]).cuda()
    nq = int(oq[-1])
    lse = torch.empty((1, nq), dtype=torch.float32, device="cuda")
    out, _ = binding.jfa_forward_cross(qd, kd, dev["v"], torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda(), 512, 512, lse=lse)
    torch.cuda.synchronize()
    out = out[:nq]
    r_out, r_lse = cross.forward(q, k, host["v"], oq, ok)
    assert np.isfinite(f64(out)).all() and np.isfinite(f64(lse)).all()
    gate_bf16("out", f64(out), r_out)
    gate_bf16("lse", f64(lse), r_lse, abs_tol=2e-2 * max(1.0, np.abs(r_lse).max() / 4))


def test_cross_full_size_on_sampled_pairs():
    """Keys with the benchmarked configuration's lengths, queries with those lengths shuffled across samples (the
    "shuffled" workload of variants_bench, B = 512, H = 8, D = 128); whole (sample, head) pairs against the oracle."""
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.synthetic import CONFIGS, lengths_for
    c = CONFIGS["c4_bimodal_bf16"]
    Lk = lengths_for(c["lengths"], c["B"], c["max_len"], np.random.Generator(np.random.PCG64(c["seed"])))
    Lq = np.random.default_rng(7).permutation(Lk)
    H, D = c["H"], c["D"]
    host, dev, oq, ok = make(Lq, Lk, H, D, "bf16", 8)
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    nq, nk = int(oq[-1]), int(ok[-1])
    nan = float("nan")   # every valid row has to be written (all samples have queries and keys): unwritten tiles stay NaN
    lse = torch.full((H, nq), nan, dtype=torch.float32, device="cuda")
    out = torch.full((nq, H, D), nan, dtype=torch.bfloat16, device="cuda")
    binding.jfa_forward_cross(dev["q"], dev["k"], dev["v"], oqd, okd, c["max_len"], c["max_len"], out=out, lse=lse)
    stats = torch.empty((2, H, nq), dtype=torch.float32, device="cuda")
    dq = torch.full((nq, H, D), nan, dtype=torch.bfloat16, device="cuda")
    dk = torch.full((nk, H, D), nan, dtype=torch.bfloat16, device="cuda")
    dv = torch.full((nk, H, D), nan, dtype=torch.bfloat16, device="cuda")
    binding.jfa_backward_cross(dev["q"], dev["k"], dev["v"], out, dev["dout"], lse, oqd, okd, c["max_len"],
                               c["max_len"], dq=dq, dk=dk, dv=dv, delta=stats)
    torch.cuda.synchronize()
    for name, t in (("out", out), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
        assert torch.isfinite(t.float()).all(), f"{name}: rows that were never written (or not finite)"
    rng = np.random.default_rng(9)
    picks = [(int(np.argmax(Lq * Lk)), 0), (int(np.argmax(Lk)), H - 1), (int(np.argmax(Lq)), 1)]
    picks += [(int(rng.integers(0, len(Lq))), int(rng.integers(0, H))) for _ in range(5)]
    for b, h in picks:
        qs, qe, ks, ke = int(oq[b]), int(oq[b + 1]), int(ok[b]), int(ok[b + 1])
        oneq = lambda x: np.ascontiguousarray(x[qs:qe, h:h + 1])
        onek = lambda x: np.ascontiguousarray(x[ks:ke, h:h + 1])
        o1q, o1k = np.array([0, qe - qs], dtype=np.int64), np.array([0, ke - ks], dtype=np.int64)
        r_out, r_lse = cross.forward(oneq(host["q"]), onek(host["k"]), onek(host["v"]), o1q, o1k)
        r_dq, r_dk, r_dv, _ = cross.backward(oneq(host["q"]), onek(host["k"]), onek(host["v"]), oneq(host["dout"]), o1q, o1k)
        tag = f"sample {b} ({qe - qs} queries, {ke - ks} keys) head {h}: "
        gate_bf16(tag + "out", f64(out[qs:qe, h:h + 1]), r_out)
        gate_bf16(tag + "lse", f64(lse[h:h + 1, qs:qe]), r_lse)
        gate_bf16(tag + "dq", f64(dq[qs:qe, h:h + 1]), r_dq, abs_tol=2e-2 * max(1.0, float(np.abs(r_dq).max()) / 2))
        gate_bf16(tag + "dk", f64(dk[ks:ke, h:h + 1]), r_dk, abs_tol=2e-2 * max(1.0, float(np.abs(r_dk).max()) / 2))
        gate_bf16(tag + "dv", f64(dv[ks:ke, h:h + 1]), r_dv, abs_tol=2e-2 * max(1.0, float(np.abs(r_dv).max()) / 2))
