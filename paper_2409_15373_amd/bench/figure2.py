#!/usr/bin/env python3
"""The four systems of the paper's Figure 2 over the maximum length, on one GPU and this library's own kernels.

    python -m paper_2409_15373_amd.bench.figure2 [--B 128] [--H 4] [--D 128] [--max-lens 128,256,...] [--reps 5]

Section 3 / Figure 2 plot latency and memory of four attention implementations against max_L in bf16:
dense attention, jagged attention, dense flash attention and jagged flash attention.  The paper's dense systems are
not available here; following its own description (the dense versions run on padded tensors), the four legs are

  dense            the unfused operators (scores -> softmax -> apply, score array in HBM) on the padded problem:
                   every sample stretched to max_L rows (offsets 0, max_L, 2 max_L, ...), i.e. B max_L^2 scores;
  jagged           the same three operators on the jagged tensor (sum L_b^2 scores): Table 1's jagged operators;
  dense flash      the fused kernel (jfa_forward / jfa_backward) on the padded problem;
  jagged flash     the fused kernel on the jagged tensor.

The padded legs do the arithmetic a padded implementation does (every padded row is computed, as in a dense kernel,
whether a mask then discards it or not); what they leave out is the jagged -> dense -> jagged conversion around
them, which `dense_compare` times.  Lengths are uniform on [1, max_L] (the recipe Table 1's FLOP ratios of 1.98 and
2.91 point to), seeded; B, H, D fixed.  Memory is what each leg has to hold at once beyond the library's O(B) table:
q, k, v, out (padded or jagged), the fp32 score array of the unfused legs, lse for the fused ones; the backward adds
dout, dq, dk, dv, and a second score array (unfused) or the two statistics planes (fused).
Prints one JSON line; per max_L the latencies in microseconds, the byte counts and the ratios the paper quotes
("up to 9x / 3x faster, 22x / 53 % less memory": context from other hardware, not a target).
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


def run_leg(lengths, H, D, max_len, fused, backward, reps):
    """Forward (and backward) latency in microseconds and the bytes held, for one leg on the given lengths."""
    import torch
    from .. import binding
    from ..synthetic import offsets_from_lengths
    n = int(lengths.sum())
    pairs = int((lengths.astype(np.int64) ** 2).sum())
    off = torch.from_numpy(offsets_from_lengths(lengths)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(0)
    mk = lambda: torch.randn(n, H, D, device="cuda", generator=gen).bfloat16()
    q, k, v = mk(), mk(), mk()
    out = torch.empty_like(q)
    values = n * H * D * 2
    r = {"rows": n, "score_pairs_per_head": pairs}
    if fused:
        lse = torch.empty(H, n, device="cuda")
        r["fwd_us"] = _time(lambda: binding.jfa_forward(q, k, v, off, max_len, out=out, lse=lse), reps)
        r["fwd_bytes"] = 4 * values + 4 * H * n
        if backward:
            dout = mk()
            dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
            stats = torch.empty(2, H, n, device="cuda")
            r["bwd_us"] = _time(lambda: binding.jfa_backward(q, k, v, out, dout, lse, off, max_len, dq=dq, dk=dk, dv=dv, delta=stats), reps)
            r["fwd_bwd_bytes"] = 8 * values + 4 * H * n + 8 * H * n
    else:
        sq = binding.jfa_square_offsets(off)
        scores = torch.empty(H * pairs, dtype=torch.float32, device="cuda")

        def fwd():
            binding.jfa_unfused_scores(q, k, off, sq, max_len, scores)
            binding.jfa_unfused_softmax(off, sq, max_len, H, scores)
            binding.jfa_unfused_apply(scores, v, off, sq, max_len, out=out)

        r["fwd_us"] = _time(fwd, reps)
        r["fwd_bytes"] = 4 * values + 4 * H * pairs
        if backward:
            dout = mk()
            dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
            dscores = torch.empty_like(scores)
            inv_sqrt_d = 1.0 / float(np.sqrt(D))

            def bwd():   # `scores` holds the probabilities of the forward
                binding.jfa_unfused_product(dout, v, off, sq, max_len, 1.0, dscores)
                binding.jfa_unfused_apply_transposed(scores, dout, off, sq, max_len, out=dv)
                binding.jfa_unfused_softmax_backward(scores, off, sq, max_len, H, inv_sqrt_d, dscores)
                binding.jfa_unfused_apply(dscores, k, off, sq, max_len, out=dq)
                binding.jfa_unfused_apply_transposed(dscores, q, off, sq, max_len, out=dk)

            r["bwd_us"] = _time(bwd, reps)
            r["fwd_bwd_bytes"] = 8 * values + 8 * H * pairs
    for key in ("fwd_us", "bwd_us"):
        if key in r:
            r[key] = round(r[key], 1)
    torch.cuda.empty_cache()
    return r


LEGS = (("dense", True, False), ("jagged", False, False), ("dense_flash", True, True), ("jagged_flash", False, True))


def sweep(B, H, D, max_lens, reps, backward=True, seed=0, budget_bytes=160e9):
    from ..synthetic import lengths_for
    points = []
    for max_len in max_lens:
        L = lengths_for("uniform", B, max_len, np.random.Generator(np.random.PCG64(seed + max_len)))
        padded = np.full(B, max_len, dtype=np.int64)
        p = {"max_L": max_len, "B": B, "H": H, "D": D, "sum_B": int(L.sum()),
             "padded_over_jagged_rows": round(float(B * max_len) / float(L.sum()), 2),
             "padded_over_jagged_pairs": round(float(B) * max_len ** 2 / float((L.astype(np.float64) ** 2).sum()), 2)}
        for name, pad, fused in LEGS:
            lens = padded if pad else L
            need = 8 * H * float((lens.astype(np.float64) ** 2).sum()) if not fused else 0.0
            if need > budget_bytes:      # the unfused score arrays of this point do not fit the memory set aside for them
                p[name] = {"skipped": f"score arrays need {need / 1e9:.1f} GB"}
                continue
            p[name] = run_leg(lens, H, D, max_len, fused, backward, reps)
        ok = lambda a: "fwd_us" in p[a]
        ratio = lambda a, b, key: round(p[a][key] / p[b][key], 2) if ok(a) and ok(b) and key in p[a] and key in p[b] else None
        p["ratios"] = {
            "latency_fwd_dense_over_jagged_flash": ratio("dense", "jagged_flash", "fwd_us"),
            "latency_fwd_dense_flash_over_jagged_flash": ratio("dense_flash", "jagged_flash", "fwd_us"),
            "latency_fwd_dense_over_jagged": ratio("dense", "jagged", "fwd_us"),
            "latency_bwd_dense_over_jagged_flash": ratio("dense", "jagged_flash", "bwd_us"),
            "latency_bwd_dense_flash_over_jagged_flash": ratio("dense_flash", "jagged_flash", "bwd_us"),
            "memory_fwd_dense_over_jagged_flash": ratio("dense", "jagged_flash", "fwd_bytes"),
            "memory_fwd_dense_over_jagged": ratio("dense", "jagged", "fwd_bytes"),
            "memory_fwd_saving_jagged_flash_vs_dense_flash": (round(1.0 - p["jagged_flash"]["fwd_bytes"] / p["dense_flash"]["fwd_bytes"], 3)
                                                              if ok("dense_flash") and ok("jagged_flash") else None),
        }
        points.append(p)
        print(f"[figure2] max_L {max_len}: " + ", ".join(f"{n} {p[n].get('fwd_us', '-')} us" for n, _, _ in LEGS), file=sys.stderr, flush=True)
    return points


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--B", type=int, default=128)
    ap.add_argument("--H", type=int, default=4)
    ap.add_argument("--D", type=int, default=128)
    ap.add_argument("--max-lens", default="128,256,512,1024,2048,4096")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--forward-only", action="store_true")
    args = ap.parse_args()
    import torch
    from .. import binding
    binding.load()
    assert torch.cuda.is_available(), "needs the GPU"
    points = sweep(args.B, args.H, args.D, [int(x) for x in args.max_lens.split(",")], args.reps, backward=not args.forward_only)
    print(json.dumps({"comparison": "the four systems of Figure 2 (dense = this library's kernels on the padded problem)",
                      "dtype": "bf16", "data": "synthetic, lengths uniform on [1, max_L]", "points": points}))


if __name__ == "__main__":
    main()
