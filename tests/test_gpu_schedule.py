"""The offsets-driven scheduler kernel against plain numpy (integer work: bit-exact where unique)."""
import numpy as np
import pytest
import torch

from paper_2409_15373_amd.synthetic import make_workload

pytestmark = pytest.mark.gpu


def check_schedule(lengths, block_rows):
    from paper_2409_15373_amd import binding
    lengths = np.asarray(lengths, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    order, tile_start = binding.jfa_build_schedule(torch.from_numpy(off).cuda(), block_rows)
    torch.cuda.synchronize()
    order = order.cpu().numpy(); tile_start = tile_start.cpu().numpy()
    B = len(lengths)
    assert sorted(order.tolist()) == list(range(B)), "order must be a permutation of the samples"
    nq = (lengths + block_rows - 1) // block_rows
    got_nq = np.diff(tile_start)
    np.testing.assert_array_equal(got_nq, nq[order])                     # each position carries its sample's block count
    bins = np.minimum(nq[order], 1023)
    assert (np.diff(bins) <= 0).all(), "samples with more row blocks come first"
    assert tile_start[0] == 0 and tile_start[-1] == nq.sum()


@pytest.mark.parametrize("block_rows", [64, 128])
def test_schedule_small_and_edge_cases(block_rows):
    check_schedule([5], block_rows)
    check_schedule([0, 0, 3, 0], block_rows)
    check_schedule([64, 65, 128, 129, 1, 127, 256], block_rows)
    check_schedule([0] * 7, block_rows)
    check_schedule(np.arange(1, 3000) % 700, block_rows)                 # B > one scan chunk, zero lengths inside


@pytest.mark.parametrize("name", ["c2_geom_bf16", "c3_zipf_bf16", "c4_bimodal_bf16"])
def test_schedule_on_named_configs(name):
    from paper_2409_15373_amd.synthetic import CONFIGS, lengths_for
    c = CONFIGS[name]
    L = lengths_for(c["lengths"], c["B"], c["max_len"], np.random.Generator(np.random.PCG64(c["seed"])))
    check_schedule(L, 128)


def test_top_bin_overflow():
    # more than 1022 row blocks per sample: all share the top bin and must still be scheduled exactly once
    check_schedule([32 * 1500, 32 * 1023, 7, 32 * 2000, 32 * 1022], 32)


def test_check_offsets_flags():
    from paper_2409_15373_amd import binding
    good = torch.tensor([0, 3, 3, 10], dtype=torch.int64).cuda()
    assert binding.jfa_check_offsets(good, 7) == 0
    assert binding.jfa_check_offsets(good, 6) == 4
    assert binding.jfa_check_offsets(torch.tensor([1, 3, 2], dtype=torch.int64).cuda(), 100) == 3


@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("bf16", 32), ("f32", 32)])
@pytest.mark.parametrize("mode", ["self", "causal", "cross"])
def test_small_problems_build_their_schedule_in_the_kernel(dtype, D, mode):
    """Problems of at most four work items per compute unit (by the bound B * blocks(max_len) * H) run without the
    scheduler launch: every workgroup builds the schedule itself.  max_len is only a bound, so the same inputs with a
    huge bound take the scheduler-kernel path; both must give the same bits, forward and backward (a tile's arithmetic
    does not depend on the order in which tiles are handed out)."""
    from paper_2409_15373_amd import binding
    rng = np.random.default_rng(17)
    B, H = 200, 2
    Lq = rng.integers(0, 257, size=B); Lq[3] = 256; Lq[10] = 0
    Lk = rng.integers(0, 257, size=B) if mode == "cross" else Lq
    oq = np.concatenate([[0], np.cumsum(Lq)]).astype(np.int64); ok = np.concatenate([[0], np.cumsum(Lk)]).astype(np.int64)
    nq, nk = int(oq[-1]), int(ok[-1])
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(5)
    mk = lambda n: torch.randn(n, H, D, device="cuda", generator=gen).to(tdt)
    q, dout, k, v = mk(nq), mk(nq), mk(nk), mk(nk)
    oqd, okd = torch.from_numpy(oq).cuda(), torch.from_numpy(ok).cuda()
    results = []
    for bound in (256, 1 << 20):       # 200 * 2 * 2 = 800 items <= 4 * 256 compute units; the huge bound is far above
        if mode == "cross":
            out, lse = binding.jfa_forward_cross(q, k, v, oqd, okd, bound, bound)
            dq, dk, dv, delta = binding.jfa_backward_cross(q, k, v, out, dout, lse, oqd, okd, bound, bound)
        else:
            out, lse = binding.jfa_forward(q, k, v, oqd, bound, causal=mode == "causal")
            dq, dk, dv, delta = binding.jfa_backward(q, k, v, out, dout, lse, oqd, bound, causal=mode == "causal")
        torch.cuda.synchronize()
        results.append((out, lse, dq, dk, dv, delta))
    for name, a, b in zip(("out", "lse", "dq", "dk", "dv", "delta"), *results):
        if mode == "cross" and name == "lse":
            a, b = torch.nan_to_num(a, neginf=-1e30), torch.nan_to_num(b, neginf=-1e30)
        assert torch.equal(a, b), f"{name} differs between the in-kernel schedule and the scheduler kernel"
