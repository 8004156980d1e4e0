"""Pins for oracle/convert.py (jagged <-> padded-dense, paper Section 2.2): checked against library routines
and properties, none of which is the oracle's own loop.

  V1  jagged_to_dense equals torch.nn.utils.rnn.pad_sequence of the per-sample slices (plus all-pad columns up to
      max_len), for zero and non-zero pad values
  V2  dense_to_jagged equals boolean-mask selection dense[mask] with mask[b, i] = i < L_b
  V3  round trip: dense_to_jagged(jagged_to_dense(x)) == x bit for bit; the padding of jagged_to_dense(dense_to_jagged(d))
      is the pad value and the rest is d
  V4  hand-written tiny case, zero-length samples, a sample of exactly max_len, and an over-long sample is an error
"""
import numpy as np
import pytest
import torch

from oracle import convert
from paper_2409_15373_amd.synthetic import offsets_from_lengths


def _values(lengths, inner, seed=0, dtype=np.float32):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((int(np.sum(lengths)),) + inner).astype(dtype)


@pytest.mark.parametrize("pad", [0.0, -7.5])
def test_v1_matches_pad_sequence(pad):
    lengths = np.array([5, 0, 9, 1, 3])
    off = offsets_from_lengths(lengths)
    x = _values(lengths, (2, 4), seed=1)
    got = convert.jagged_to_dense(x, off, 12, pad)
    pieces = [torch.from_numpy(x[off[b]:off[b + 1]]) for b in range(len(lengths))]
    ref = torch.nn.utils.rnn.pad_sequence(pieces, batch_first=True, padding_value=pad).numpy()   # [B, 9, 2, 4]
    assert got.shape == (5, 12, 2, 4)
    np.testing.assert_array_equal(got[:, :9], ref)
    np.testing.assert_array_equal(got[:, 9:], np.float32(pad))


def test_v2_matches_mask_selection():
    lengths = np.array([4, 7, 0, 2])
    off = offsets_from_lengths(lengths)
    d = np.random.default_rng(2).standard_normal((4, 7, 3, 2)).astype(np.float32)
    mask = np.arange(7)[None, :] < lengths[:, None]
    np.testing.assert_array_equal(convert.dense_to_jagged(d, off), torch.from_numpy(d)[torch.from_numpy(mask)].numpy())


def test_v3_round_trips():
    lengths = np.array([6, 1, 0, 8, 8, 3])
    off = offsets_from_lengths(lengths)
    x = _values(lengths, (3, 8), seed=3).view(np.uint32)                  # compare bit patterns
    np.testing.assert_array_equal(convert.dense_to_jagged(convert.jagged_to_dense(x, off, 8, 0), off), x)
    d = np.random.default_rng(4).standard_normal((6, 8, 5)).astype(np.float32)
    back = convert.jagged_to_dense(convert.dense_to_jagged(d, off), off, 8, 99.0)
    mask = np.arange(8)[None, :] < lengths[:, None]
    np.testing.assert_array_equal(back[mask], d[mask])
    np.testing.assert_array_equal(back[~mask], np.float32(99.0))


def test_v4_tiny_by_hand_and_errors():
    x = np.array([[1, 2], [3, 4], [5, 6]], dtype=np.int16)                # samples: [row0, row1], [], [row2]
    off = np.array([0, 2, 2, 3])
    d = convert.jagged_to_dense(x, off, 2, -1)
    assert d.tolist() == [[[1, 2], [3, 4]], [[-1, -1], [-1, -1]], [[5, 6], [-1, -1]]]
    assert convert.dense_to_jagged(d, off).tolist() == x.tolist()
    with pytest.raises(ValueError):
        convert.jagged_to_dense(x, off, 1, 0)
    with pytest.raises(ValueError):
        convert.dense_to_jagged(d[:, :1], off)
