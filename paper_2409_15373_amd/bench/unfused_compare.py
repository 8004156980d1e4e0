#!/usr/bin/env python3
"""Fused jagged flash attention versus the unfused jagged attention, forward and backward, on the same GPU.

    python -m paper_2409_15373_amd.bench.unfused_compare [--workloads c2_geom_bf16,c3_zipf_bf16,...] [--reps N]

The paper's Section 3 compares the fused kernel with "jagged attention": the three jagged operators of its
Table 1 run one after another, with the L_b x L_b score blocks of every sample and head written to memory
between them.  Both sides here are this library's own kernels (jfa_forward against jfa_unfused_scores ->
jfa_unfused_softmax -> jfa_unfused_apply).  For each workload it reports microseconds per call of either side,
the three operators' own durations (HIP events inside the library) with the rate at which each moves the
score array (4 bytes per score: written once by scores, read and written by softmax, read by apply), and the
extra device memory either side needs beyond q, k, v and out (Section 3's memory claim): the fp32 score array
for the unfused path, the fp32 log-sum-exp rows for the fused one.  The backward is compared the same way:
jfa_backward against product (dP), apply_transposed (dV), softmax_backward (dS), apply (dQ), apply_transposed (dK),
which need a second array of that size.
Inputs are random normals of the workload's scale drawn on the device.  Prints one JSON line.
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", default="c2_geom_bf16,c3_zipf_bf16,c4_bimodal_bf16,c5_uniform_bf16")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from .. import binding
    from ..synthetic import CONFIGS, lengths_for, offsets_from_lengths
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    result = {"comparison": "fused jagged flash attention vs unfused jagged attention (scores, softmax, apply and their backward operators)",
              "dtype": "bf16", "data": "synthetic", "workloads": {}}
    for name in args.workloads.split(","):
        c = CONFIGS[name]
        H, D, max_len = c["H"], c["D"], c["max_len"]
        L = lengths_for(c["lengths"], c["B"], max_len, np.random.Generator(np.random.PCG64(c["seed"])))
        n = int(L.sum())
        pairs = int((L.astype(np.int64) ** 2).sum())
        off = torch.from_numpy(offsets_from_lengths(L)).cuda()
        gen = torch.Generator(device="cuda").manual_seed(0)
        mk = lambda s: (torch.randn(n, H, D, device="cuda", generator=gen) * s).bfloat16()
        q, k, v = mk(c["sigma"]), mk(c["sigma"]), mk(1.0)
        out, lse = torch.empty_like(q), torch.empty(H, n, device="cuda")
        out_u = torch.empty_like(q)
        sq = binding.jfa_square_offsets(off)
        assert int(sq[-1].item()) == pairs
        scores = torch.empty(H * pairs, dtype=torch.float32, device="cuda")

        def fused():
            binding.jfa_forward(q, k, v, off, max_len, out=out, lse=lse)

        def unfused():
            binding.jfa_unfused_scores(q, k, off, sq, max_len, scores)
            binding.jfa_unfused_softmax(off, sq, max_len, H, scores)
            binding.jfa_unfused_apply(scores, v, off, sq, max_len, out=out_u)

        dout = mk(1.0)
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        dq_u, dk_u, dv_u = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        stats = torch.empty(2, H, n, device="cuda")
        dscores = torch.empty_like(scores)
        inv_sqrt_d = 1.0 / float(np.sqrt(D))

        def fused_bwd():
            binding.jfa_backward(q, k, v, out, dout, lse, off, max_len, dq=dq, dk=dk, dv=dv, delta=stats)

        def unfused_bwd():   # `scores` holds the probabilities of the last unfused forward
            binding.jfa_unfused_product(dout, v, off, sq, max_len, 1.0, dscores)
            binding.jfa_unfused_apply_transposed(scores, dout, off, sq, max_len, out=dv_u)
            binding.jfa_unfused_softmax_backward(scores, off, sq, max_len, H, inv_sqrt_d, dscores)
            binding.jfa_unfused_apply(dscores, k, off, sq, max_len, out=dq_u)
            binding.jfa_unfused_apply_transposed(dscores, q, off, sq, max_len, out=dk_u)

        t_f = _time(fused, args.reps)
        t_u = _time(unfused, args.reps)
        t_fb = _time(fused_bwd, args.reps)
        t_ub = _time(unfused_bwd, args.reps)
        diff_b = max((a.float() - b.float()).abs().max().item() for a, b in ((dq, dq_u), (dk, dk_u), (dv, dv_u)))
        binding.jfa_timing_enable(True)
        binding.jfa_timing_read()
        for _ in range(args.reps):
            unfused()
        torch.cuda.synchronize()
        timers = binding.jfa_timing_read()
        binding.jfa_timing_enable(False)
        diff = (out.float() - out_u.float()).abs().max().item()
        score_bytes = 4 * H * pairs
        ops = {}
        for op, passes in (("unfused_scores", 1), ("unfused_softmax", 2), ("unfused_apply", 1)):
            ms, cnt = timers[op]
            us = ms * 1e3 / cnt
            ops[op] = {"us": round(us, 1), "score_array_GB_per_s": round(passes * score_bytes / (us * 1e-6) / 1e9, 1)}
        result["workloads"][name] = {
            "B": c["B"], "H": H, "D": D, "max_len": max_len, "rows": n, "score_pairs_per_head": pairs,
            "fused_us": round(t_f, 1), "unfused_us": round(t_u, 1), "speedup": round(t_u / t_f, 2),
            "fused_bwd_us": round(t_fb, 1), "unfused_bwd_us": round(t_ub, 1), "speedup_bwd": round(t_ub / t_fb, 2),
            "max_abs_difference_of_gradients": round(diff_b, 5),
            "operators": ops,
            "fused_extra_bytes": 4 * H * n, "unfused_extra_bytes": score_bytes,
            "qkvo_bytes": 4 * n * H * D * 2,
            "memory_saving": round(1.0 - (4 * n * H * D * 2 + 4 * H * n) / (4 * n * H * D * 2 + score_bytes), 3),
            "max_abs_difference_of_outputs": round(diff, 5),
        }
        print(f"[unfused_compare] {name}: forward fused {t_f:.1f} us, unfused {t_u:.1f} us ({t_u / t_f:.2f}x); backward "
              f"fused {t_fb:.1f} us, unfused {t_ub:.1f} us ({t_ub / t_fb:.2f}x); score array {score_bytes / 1e9:.2f} GB",
              file=sys.stderr, flush=True)
        del scores, dscores, q, k, v, out, out_u, lse, dout, dq, dk, dv, dq_u, dk_u, dv_u
        torch.cuda.empty_cache()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
