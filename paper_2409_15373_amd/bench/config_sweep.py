#!/usr/bin/env python3
"""Microseconds per call and useful TFLOP/s of the forward and of forward + backward on all five configurations.

    python -m paper_2409_15373_amd.bench.config_sweep [--configs c1_tiny_f32,...] [--repeats 5]

Per configuration: >= 10 warm-up calls, then the median over `repeats` timings of N back-to-back calls on one
stream bracketed by HIP events (N chosen so that one timing lasts >= 50 ms).  A call is everything the entry point
enqueues (scheduler + kernels).  Useful flops: 4 H D sum(L^2) forward, 14 H D sum(L^2) forward + backward, from the
realised offsets.  Configurations whose tensors fit in the 256 MB Infinity Cache (c1, c2) are also timed cache-cold:
the calls rotate over enough distinct copies of the inputs and outputs to cover more than 512 MB, so no call finds
its data in a cache.  Inputs are random normals of the configuration's scale drawn on the device (timings do not
depend on the values; the parity tests use the seeded host-side data).  Prints one JSON line.
"""
import argparse
import json
import statistics
import sys

import numpy as np

PEAK_TFLOPS = 2516.6


def _timed(fn, n):
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(n):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def _median_us(fn, repeats):
    import torch
    for i in range(10):
        fn(i)
    torch.cuda.synchronize()
    one = _timed(fn, 10)
    n = max(10, int(50e3 / max(one, 1e-3)) + 1)
    return statistics.median(_timed(fn, n) for _ in range(repeats)), n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="c1_tiny_f32,c2_geom_bf16,c3_zipf_bf16,c4_bimodal_bf16,c5_uniform_bf16")
    ap.add_argument("--repeats", type=int, default=5)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import CONFIGS, lengths_for, offsets_from_lengths
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    result = {"data": "synthetic", "peak_bf16_TFLOP_per_s": PEAK_TFLOPS, "configs": {}}
    for name in args.configs.split(","):
        c = CONFIGS[name]
        B, H, D, max_len = c["B"], c["H"], c["D"], c["max_len"]
        dt = torch.float32 if c["dtype"] == "f32" else torch.bfloat16
        L = lengths_for(c["lengths"], B, max_len, np.random.Generator(np.random.PCG64(c["seed"])))
        n = int(L.sum())
        S2 = float((L.astype(np.float64) ** 2).sum())
        off = torch.from_numpy(offsets_from_lengths(L)).cuda()
        footprint = 8 * n * H * D * (4 if dt == torch.float32 else 2)        # q, k, v, out, dout, dq, dk, dv
        copies = 1 if footprint >= 256e6 else int(512e6 // footprint) + 2
        planes = 1 if dt == torch.float32 else 2
        gen = torch.Generator(device="cuda").manual_seed(0)

        def mk(s):
            return (torch.randn(copies, n, H, D, device="cuda", generator=gen) * s).to(dt)

        q, k, v, dout = mk(c["sigma"]), mk(c["sigma"]), mk(1.0), mk(1.0)
        out, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
        def per_copy(*shape):   # one contiguous fp32 block per copy, each starting on a 256-byte boundary
            size = int(np.prod(shape))
            stride = (size + 63) // 64 * 64
            flat = torch.empty(copies * stride, device="cuda")
            return [flat[j * stride: j * stride + size].view(*shape) for j in range(copies)]

        lse, stats = per_copy(H, n), per_copy(planes, H, n)

        def fwd(i, m=1):
            j = i % m
            binding.jfa_forward(q[j], k[j], v[j], off, max_len, out=out[j], lse=lse[j])

        def step(i, m=1):
            j = i % m
            binding.jfa_forward(q[j], k[j], v[j], off, max_len, out=out[j], lse=lse[j])
            binding.jfa_backward(q[j], k[j], v[j], out[j], dout[j], lse[j], off, max_len, dq=dq[j], dk=dk[j], dv=dv[j], delta=stats[j])

        r = {"B": B, "H": H, "D": D, "max_len": max_len, "dtype": c["dtype"], "sum_B": n, "S2": S2}
        for tag, fn, flops in (("fwd", fwd, 4.0 * H * D * S2), ("fwd_bwd", step, 14.0 * H * D * S2)):
            us, calls = _median_us(lambda i: fn(i, 1), args.repeats)
            r[tag + "_us"] = round(us, 2)
            r[tag + "_calls_per_timing"] = calls
            r[tag + "_useful_TFLOP_per_s"] = round(flops / us / 1e6, 2)
            if c["dtype"] == "bf16":
                r[tag + "_pct_bf16_mfma_peak"] = round(100.0 * flops / us / 1e6 / PEAK_TFLOPS, 2)
            if copies > 1:
                us_cold, _ = _median_us(lambda i: fn(i, copies), args.repeats)
                r[tag + "_us_cache_cold"] = round(us_cold, 2)
        if copies > 1:
            r["cache_cold_copies"] = copies
        result["configs"][name] = r
        print(f"[config_sweep] {name}: " + ", ".join(f"{k}={v}" for k, v in r.items() if k.endswith("_us") or k.endswith("cold") or k.endswith("peak")),
              file=sys.stderr, flush=True)
        del q, k, v, dout, out, dq, dk, dv, lse, stats
        torch.cuda.empty_cache()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
