#!/usr/bin/env python3
"""The unfused forward operators next to the framework's plain streaming kernels on the same score array.

    python -m paper_2409_15373_amd.bench.unfused_memory_probe [--workload c4_bimodal_bf16] [--reps 2]

Meant to run under rocprofv3 (kernel trace, or one --pmc pass of memory counters): per repetition it launches
jfa_unfused_scores (writes the fp32 score array once), jfa_unfused_softmax (reads and writes it), jfa_unfused_apply
(reads it), and then three torch kernels over the very same array as yardsticks of what a plain stream reaches on
this machine: `mul_` (read + write), `sum` (read), `fill_` (write).  Prints the array's size; the durations and
counters come from the profiler.  Inputs are random normals drawn on the device.
"""
import argparse

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c4_bimodal_bf16")
    ap.add_argument("--reps", type=int, default=2)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import CONFIGS, lengths_for, offsets_from_lengths
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    c = CONFIGS[args.workload]
    H, D, max_len = c["H"], c["D"], c["max_len"]
    L = lengths_for(c["lengths"], c["B"], max_len, np.random.Generator(np.random.PCG64(c["seed"])))
    n = int(L.sum())
    pairs = int((L.astype(np.int64) ** 2).sum())
    off = torch.from_numpy(offsets_from_lengths(L)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(0)
    mk = lambda: torch.randn(n, H, D, device="cuda", generator=gen).bfloat16()
    q, k, v = mk(), mk(), mk()
    out = torch.empty_like(q)
    sq = binding.jfa_square_offsets(off)
    scores = torch.empty(H * pairs, dtype=torch.float32, device="cuda")
    for _ in range(args.reps):
        binding.jfa_unfused_scores(q, k, off, sq, max_len, scores)
        binding.jfa_unfused_softmax(off, sq, max_len, H, scores)
        binding.jfa_unfused_apply(scores, v, off, sq, max_len, out=out)
        scores.mul_(1.0)
        scores.sum()
        scores.fill_(0.5)
    torch.cuda.synchronize()
    print(f"{args.workload}: score array {4 * H * pairs} bytes, {args.reps} repetitions")


if __name__ == "__main__":
    main()
