#!/usr/bin/env python3
"""Timing of the cross and causal variants of jagged attention against the bf16 MFMA roofline.

    python -m paper_2409_15373_amd.bench.variants_bench [--reps N]

The paper's feature interaction attends from a sample's target items to its feature values: few queries, many
keys.  Three synthetic workloads with B = 512, H = 8, D = 128 and the keys' lengths of the benchmarked self-attention
configuration (bimodal, up to 4096): queries uniform on [1, 32] ("few_targets": the backward is the one-pass kernel
for at most 32 queries per sample, bound by reading K and V and writing dK and dV once), queries uniform on [1, 256]
("targets"), and queries with the keys' lengths shuffled across samples ("shuffled": as much work as self attention,
but L_q != L_kv in every sample).  Useful flops: 4 H D sum(L_q L_kv) forward, 10 H D sum(L_q L_kv) backward;
algorithmic bytes: every input row read once and every output row written once (forward: Q, K, V, out; backward:
Q, K, V, out, dO, dQ, dK, dV; bf16; the fp32 statistics are not counted).  A fourth workload runs causal self
attention (jfa_forward_causal / jfa_backward_causal) on that configuration itself: sum L (L + 1) / 2 query-key
pairs per head.  Prints one JSON line.
"""
import argparse
import json

import numpy as np

PEAK_TFLOPS = 2516.6


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import CONFIGS, lengths_for, offsets_from_lengths
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    c = CONFIGS["c4_bimodal_bf16"]
    B, H, D = c["B"], c["H"], c["D"]
    rng = np.random.Generator(np.random.PCG64(c["seed"]))
    Lk = lengths_for(c["lengths"], B, c["max_len"], rng)
    cases = {"targets": (lengths_for("uniform", B, 256, rng), 256), "shuffled": (rng.permutation(Lk), c["max_len"]),
             "few_targets": (lengths_for("uniform", B, 32, rng), 32)}
    result = {"dtype": "bf16", "data": "synthetic", "B": B, "H": H, "D": D, "bound": "mfma", "peak_TFLOP_per_s": PEAK_TFLOPS, "workloads": {}}
    gen = torch.Generator(device="cuda").manual_seed(0)
    for name, (Lq, max_q) in cases.items():
        nq, nk = int(Lq.sum()), int(Lk.sum())
        pairs = float((Lq.astype(np.float64) * Lk).sum())
        oq, ok = (torch.from_numpy(offsets_from_lengths(x)).cuda() for x in (Lq, Lk))
        mk = lambda n, s: (torch.randn(n, H, D, device="cuda", generator=gen) * s).bfloat16()
        q, k, v, dout = mk(nq, c["sigma"]), mk(nk, c["sigma"]), mk(nk, 1.0), mk(nq, 1.0)
        out, lse = torch.empty_like(q), torch.empty(H, nq, device="cuda")
        dq, dk, dv, stats = torch.empty_like(q), torch.empty_like(k), torch.empty_like(k), torch.empty(2, H, nq, device="cuda")
        fwd = lambda: binding.jfa_forward_cross(q, k, v, oq, ok, max_q, c["max_len"], out=out, lse=lse)
        bwd = lambda: binding.jfa_backward_cross(q, k, v, out, dout, lse, oq, ok, max_q, c["max_len"], dq=dq, dk=dk, dv=dv, delta=stats)
        t_f, t_b = _time(fwd, args.reps), _time(bwd, args.reps)
        f_f, f_b = 4.0 * H * D * pairs, 10.0 * H * D * pairs
        row = 2.0 * H * D   # bytes of one bf16 row of all heads
        by_f, by_b = row * (2 * nq + 2 * nk), row * (4 * nq + 4 * nk)
        result["workloads"][name] = {
            "sum_Bq": nq, "sum_Bkv": nk, "query_key_pairs_per_head": pairs,
            "fwd_us": round(t_f, 1), "fwd_TFLOP_per_s": round(f_f / t_f / 1e6, 1), "fwd_frac_of_peak": round(f_f / t_f / 1e6 / PEAK_TFLOPS, 3),
            "bwd_us": round(t_b, 1), "bwd_useful_TFLOP_per_s": round(f_b / t_b / 1e6, 1), "bwd_frac_of_peak": round(f_b / t_b / 1e6 / PEAK_TFLOPS, 3),
            "fwd_algorithmic_TB_per_s": round(by_f / t_f / 1e6, 2), "bwd_algorithmic_TB_per_s": round(by_b / t_b / 1e6, 2),
        }
    # causal self attention on the benchmarked configuration
    n = int(Lk.sum())
    pairs = float((Lk.astype(np.float64) * (Lk + 1) / 2).sum())
    off = torch.from_numpy(offsets_from_lengths(Lk)).cuda()
    mk = lambda s: (torch.randn(n, H, D, device="cuda", generator=gen) * s).bfloat16()
    q, k, v, dout = mk(c["sigma"]), mk(c["sigma"]), mk(1.0), mk(1.0)
    out, lse = torch.empty_like(q), torch.empty(H, n, device="cuda")
    dq, dk, dv, stats = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty(2, H, n, device="cuda")
    fwd = lambda: binding.jfa_forward(q, k, v, off, c["max_len"], out=out, lse=lse, causal=True)
    bwd = lambda: binding.jfa_backward(q, k, v, out, dout, lse, off, c["max_len"], dq=dq, dk=dk, dv=dv, delta=stats, causal=True)
    t_f, t_b = _time(fwd, args.reps), _time(bwd, args.reps)
    f_f, f_b = 4.0 * H * D * pairs, 10.0 * H * D * pairs
    result["workloads"]["causal"] = {
        "sum_B": n, "query_key_pairs_per_head": pairs,
        "fwd_us": round(t_f, 1), "fwd_TFLOP_per_s": round(f_f / t_f / 1e6, 1), "fwd_frac_of_peak": round(f_f / t_f / 1e6 / PEAK_TFLOPS, 3),
        "bwd_us": round(t_b, 1), "bwd_useful_TFLOP_per_s": round(f_b / t_b / 1e6, 1), "bwd_frac_of_peak": round(f_b / t_b / 1e6 / PEAK_TFLOPS, 3),
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
