#!/usr/bin/env python3
"""Jagged versus padded-dense attention on the same GPU and the same kernels.

    python -m paper_2409_15373_amd.bench.dense_compare [--workloads c2_geom_bf16,c3_zipf_bf16,...] [--reps N]

The paper's Section 3 / Figure 2 compares jagged flash attention with dense flash attention on padded
tensors as a function of the maximum length.  The comparison systems themselves are not available here, so
the dense side is this library run on the padded problem: every sample stretched to max_len (offsets =
0, max_len, 2 max_len, ...), which is exactly what a dense [B, max_len, H, D] flash-attention call computes.
For each workload it reports microseconds per call of forward and of forward + backward for both shapes,
their ratio, and the ratio of the values-tensor footprints (Section 3's memory claim).  It also times the two
conversions a padded pipeline needs around its dense operators (Section 2.2): jfa_jagged_to_dense and
jfa_dense_to_jagged on one values tensor, with the rate at which they move their algorithmic bytes (the jagged
rows once, plus the whole dense tensor on the way out).  Inputs are random normals of the workload's scale
drawn on the device; timings do not depend on the values.
Prints one JSON line.
"""
import argparse
import json
import sys

import numpy as np


def _time(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def _run(lengths, H, D, sigma, max_len, reps):
    import torch
    from .. import binding
    from ..synthetic import offsets_from_lengths
    n = int(lengths.sum())
    off = torch.from_numpy(offsets_from_lengths(lengths)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(0)
    mk = lambda s: (torch.randn(n, H, D, device="cuda", generator=gen) * s).bfloat16()
    q, k, v, dout = mk(sigma), mk(sigma), mk(1.0), mk(1.0)
    out, lse = torch.empty_like(q), torch.empty(H, n, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    stats = torch.empty(2, H, n, device="cuda")
    fwd = lambda: binding.jfa_forward(q, k, v, off, max_len, out=out, lse=lse)
    bwd = lambda: binding.jfa_backward(q, k, v, out, dout, lse, off, max_len, dq=dq, dk=dk, dv=dv, delta=stats)
    t_f = _time(fwd, reps)
    t_b = _time(bwd, reps)
    return {"rows": n, "fwd_us": round(t_f, 1), "fwd_bwd_us": round(t_f + t_b, 1), "values_tensor_bytes": n * H * D * 2}


def _conversions(lengths, H, D, max_len, reps):
    import torch
    from .. import binding
    from ..synthetic import offsets_from_lengths
    n, B = int(lengths.sum()), len(lengths)
    off = torch.from_numpy(offsets_from_lengths(lengths)).cuda()
    x = torch.randn(n, H, D, device="cuda").bfloat16()
    dense = torch.empty(B, max_len, H, D, device="cuda", dtype=torch.bfloat16)
    back = torch.empty_like(x)
    t_pad = _time(lambda: binding.jfa_jagged_to_dense(x, off, max_len, 0.0, dense=dense), reps)
    t_unpad = _time(lambda: binding.jfa_dense_to_jagged(dense, off, back), reps)
    assert torch.equal(back.view(torch.int16), x.view(torch.int16))
    row = H * D * 2
    return {"jagged_to_dense_us": round(t_pad, 1), "jagged_to_dense_GB_per_s": round((n + B * max_len) * row / t_pad / 1e3, 1),
            "dense_to_jagged_us": round(t_unpad, 1), "dense_to_jagged_GB_per_s": round(2 * n * row / t_unpad / 1e3, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", default="c2_geom_bf16,c3_zipf_bf16,c4_bimodal_bf16,c5_uniform_bf16")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import CONFIGS, lengths_for
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    result = {"comparison": "jagged vs padded-dense (every sample stretched to max_len) on the same kernels",
              "dtype": "bf16", "data": "synthetic", "workloads": {}}
    for name in args.workloads.split(","):
        c = CONFIGS[name]
        L = lengths_for(c["lengths"], c["B"], c["max_len"], np.random.Generator(np.random.PCG64(c["seed"])))
        jag = _run(L, c["H"], c["D"], c["sigma"], c["max_len"], args.reps)
        torch.cuda.empty_cache()
        dense_L = np.full(c["B"], c["max_len"], dtype=L.dtype)
        den = _run(dense_L, c["H"], c["D"], c["sigma"], c["max_len"], max(1, args.reps // 2))
        torch.cuda.empty_cache()
        conv = _conversions(L, c["H"], c["D"], c["max_len"], args.reps)
        torch.cuda.empty_cache()
        result["workloads"][name] = {
            "B": c["B"], "H": c["H"], "D": c["D"], "max_len": c["max_len"],
            "padded_over_jagged_rows": round(den["rows"] / jag["rows"], 2),
            "padded_over_jagged_pairs": round(float(c["B"]) * c["max_len"] ** 2 / float((L.astype(np.float64) ** 2).sum()), 2),
            "jagged": jag, "dense": den,
            "speedup_fwd": round(den["fwd_us"] / jag["fwd_us"], 2),
            "speedup_fwd_bwd": round(den["fwd_bwd_us"] / jag["fwd_bwd_us"], 2),
            "memory_saving": round(1.0 - jag["values_tensor_bytes"] / den["values_tensor_bytes"], 3),
            "conversion": conv,
        }
        print(f"[dense_compare] {name}: fwd {jag['fwd_us']} vs {den['fwd_us']} us, fwd+bwd {jag['fwd_bwd_us']} vs "
              f"{den['fwd_bwd_us']} us", file=sys.stderr, flush=True)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
