"""CPU oracle for the jagged <-> padded-dense conversions (paper Section 2.2) -- test infrastructure only.

The paper's pipeline pads jagged tensors to dense ones where a dense operator is needed and strips the padding
afterwards.  With s_b = offsets[b] and L_b = offsets[b + 1] - offsets[b] <= max_len:

  jagged_to_dense(values, offsets, max_len, pad)   dense[b, i, ...] = values[s_b + i, ...] for i < L_b, pad otherwise
  dense_to_jagged(dense, offsets)                  values[s_b + i, ...] = dense[b, i, ...] for i < L_b

Both are pure data movement: the results are bit patterns of the inputs (or of `pad` cast to the input dtype), so
the comparison with the GPU is exact.  Written as the definition, one sample at a time.
"""
from __future__ import annotations

import numpy as np


def jagged_to_dense(values: np.ndarray, offsets, max_len: int, pad=0) -> np.ndarray:
    values = np.asarray(values)
    offsets = np.asarray(offsets, dtype=np.int64)
    B = len(offsets) - 1
    dense = np.empty((B, max_len) + values.shape[1:], dtype=values.dtype)
    dense[...] = np.asarray(pad).astype(values.dtype)
    for b in range(B):
        s, e = int(offsets[b]), int(offsets[b + 1])
        if e - s > max_len:
            raise ValueError(f"sample {b} is longer than max_len")
        for i in range(e - s):
            dense[b, i] = values[s + i]
    return dense


def dense_to_jagged(dense: np.ndarray, offsets) -> np.ndarray:
    dense = np.asarray(dense)
    offsets = np.asarray(offsets, dtype=np.int64)
    B = len(offsets) - 1
    values = np.empty((int(offsets[-1]),) + dense.shape[2:], dtype=dense.dtype)
    for b in range(B):
        s, e = int(offsets[b]), int(offsets[b + 1])
        if e - s > dense.shape[1]:
            raise ValueError(f"sample {b} is longer than the dense tensor")
        for i in range(e - s):
            values[s + i] = dense[b, i]
    return values
