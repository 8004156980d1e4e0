#!/usr/bin/env python3
"""Timing of the jagged feature operators of the paper's Table 1 against the HBM roofline.

    python -m paper_2409_15373_amd.bench.feature_ops_bench [--B 16384] [--max-len 512] [--D 64] [--T 64] [--reps 10]

Lengths are uniform on [1, max_len] (Table 1's jagged versions do about half the padded work, i.e. a mean length
of about max_len / 2), values random normals drawn on the device.  For every operator it reports microseconds per
call (HIP events inside the library) and the rate at which it moves its algorithmic bytes -- each input and output
tensor once: all four operators are bound by HBM (peak 8 TB/s), with 2 D T / (2 (D + T)) flops per byte at most.
Prints one JSON line.
"""
import argparse
import json

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--B", type=int, default=16384)
    ap.add_argument("--max-len", type=int, default=512)
    ap.add_argument("--D", type=int, default=64)
    ap.add_argument("--T", type=int, default=64)
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import lengths_for, offsets_from_lengths
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    B, N, D, T = args.B, args.max_len, args.D, args.T
    L = lengths_for("uniform", B, N, np.random.Generator(np.random.PCG64(0)))
    n = int(L.sum())
    off = torch.from_numpy(offsets_from_lengths(L)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(0)
    mk = lambda *shape: torch.randn(*shape, device="cuda", generator=gen).bfloat16()
    x, y, w, dy = mk(n, D), mk(n, T), mk(B, D, T), mk(n, D)
    out_t, out_w, sm, dx = torch.empty(n, T, device="cuda", dtype=torch.bfloat16), torch.empty_like(w), torch.empty_like(x), torch.empty_like(x)
    calls = {
        "jagged_dense_bmm": (lambda: binding.jfa_jagged_dense_bmm(x, w, off, N, out=out_t), 2 * (n * D + B * D * T + n * T), 2 * n * D * T),
        "jagged_jagged_bmm": (lambda: binding.jfa_jagged_jagged_bmm(x, y, off, N, out=out_w), 2 * (n * D + n * T + B * D * T), 2 * n * D * T),
        "jagged_softmax": (lambda: binding.jfa_jagged_softmax(x, off, N, y=sm), 2 * 2 * n * D, 0),
        "jagged_softmax_bwd": (lambda: binding.jfa_jagged_softmax_backward(sm, dy, off, N, dx=dx), 2 * 3 * n * D, 0),
    }
    for fn, _, _ in calls.values():
        fn()
    torch.cuda.synchronize()
    binding.jfa_timing_enable(True)
    binding.jfa_timing_read()
    for _ in range(args.reps):
        for fn, _, _ in calls.values():
            fn()
    torch.cuda.synchronize()
    timers = binding.jfa_timing_read()
    binding.jfa_timing_enable(False)
    ops = {}
    for name, (_, nbytes, flops) in calls.items():
        ms, cnt = timers[name]
        us = ms * 1e3 / cnt
        ops[name] = {"us": round(us, 1), "algorithmic_MB": round(nbytes / 1e6, 1), "GB_per_s": round(nbytes / us / 1e3, 1),
                     "frac_of_8TBps": round(nbytes / us / 1e3 / 8000.0, 3), "TFLOP_per_s": round(flops / us / 1e6, 1)}
    print(json.dumps({"workload": {"B": B, "max_len": N, "D": D, "T": T, "sum_B": n, "lengths": "uniform[1, max_len]"},
                      "dtype": "bf16", "data": "synthetic", "bound": "hbm", "operators": ops}))


if __name__ == "__main__":
    main()
