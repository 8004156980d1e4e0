"""Jagged <-> padded-dense conversion on the GPU vs oracle/convert.py: pure data movement, compared bit for bit.
Guard regions around every output must stay untouched."""
import numpy as np
import pytest
import torch

from oracle import convert
from paper_2409_15373_amd.synthetic import offsets_from_lengths, make_workload

pytestmark = pytest.mark.gpu

CASES = [
    # lengths, max_len, inner shape, dtype
    ([5, 0, 33, 1, 16, 17, 40], 40, (8, 128), torch.bfloat16),     # 2 KB rows; ends inside tiles, a full-length sample
    ([3, 7, 0, 0, 2], 7, (2, 64), torch.bfloat16),                  # max_len below the 16-row tile: tiles span samples
    ([100, 31, 64], 128, (3, 32), torch.float32),                   # fp32, 384-byte rows
    ([1] * 50, 1, (1, 32), torch.bfloat16),                         # max_len = 1
    ([0, 0, 0], 5, (2, 32), torch.bfloat16),                        # nothing but padding
    ([9, 4], 9, (8,), torch.float32),                               # 32-byte rows (two chunks)
]


def _bits(t):
    return t.cpu().view(torch.int16 if t.element_size() == 2 else torch.int32).numpy()


@pytest.mark.parametrize("lengths,max_len,inner,dtype", CASES)
@pytest.mark.parametrize("pad", [0.0, -3.5])
def test_conversions_match_the_oracle(lengths, max_len, inner, dtype, pad):
    from paper_2409_15373_amd import binding
    off = offsets_from_lengths(np.array(lengths))
    n, B = int(off[-1]), len(lengths)
    g = torch.Generator().manual_seed(7)
    x = torch.randn((n,) + inner, generator=g).to(dtype)
    guard = 3
    offd = torch.from_numpy(off).cuda()
    xd = torch.cat([x, torch.full((guard,) + inner, float("nan"), dtype=dtype)]).cuda()   # rows past sum_B: never read
    buf = torch.full((B * max_len + guard,) + inner, 777.0, dtype=dtype, device="cuda")
    dense = buf[:B * max_len].view((B, max_len) + inner)
    binding.jfa_jagged_to_dense(xd, offd, max_len, pad, dense=dense)
    torch.cuda.synchronize()
    ref = convert.jagged_to_dense(_bits(x), off, max_len, _bits(torch.tensor([pad], dtype=dtype))[0])
    np.testing.assert_array_equal(_bits(dense), ref)
    assert (buf[B * max_len:] == 777.0).all()
    # and back, from a dense tensor whose padding is not the pad value (it must not leak)
    d = torch.randn((B, max_len) + inner, generator=g).to(dtype)
    vbuf = torch.full((n + guard,) + inner, 555.0, dtype=dtype, device="cuda")
    binding.jfa_dense_to_jagged(d.cuda(), offd, vbuf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_bits(vbuf[:n]), convert.dense_to_jagged(_bits(d), off))
    assert (vbuf[n:] == 555.0).all()


def test_round_trip_on_the_zipf_workload():
    """c3 (B = 1024, max_len = 1024, H = 4, D = 128): jagged -> dense -> jagged returns the input bit for bit, the
    dense tensor equals the oracle's on sampled samples and is the pad value on every padded row."""
    from paper_2409_15373_amd import binding
    w = make_workload("c3_zipf_bf16")
    x = torch.from_numpy(w.bits["q"].view(np.int16)).view(torch.bfloat16)
    xd, offd = x.cuda(), torch.from_numpy(w.offsets).cuda()
    dense = binding.jfa_jagged_to_dense(xd, offd, w.max_len, 1.25)
    back = torch.full_like(xd, 9.0)
    binding.jfa_dense_to_jagged(dense, offd, back)
    torch.cuda.synchronize()
    assert torch.equal(back.view(torch.int16), xd.view(torch.int16))
    mask = torch.arange(w.max_len, device="cuda")[None, :] < torch.from_numpy(w.lengths).cuda()[:, None]
    assert (dense[~mask] == 1.25).all()
    order = np.argsort(w.lengths)
    for b in [int(order[-1]), int(order[0]), int(order[len(order) // 2]), 17, 1000]:
        ref = convert.jagged_to_dense(w.bits["q"][w.offsets[b]:w.offsets[b + 1]].view(np.int16), np.array([0, w.lengths[b]]),
                                      w.max_len, _bits(torch.tensor([1.25], dtype=torch.bfloat16))[0])
        np.testing.assert_array_equal(_bits(dense[b:b + 1]), ref)
