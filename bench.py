#!/usr/bin/env python3
"""Benchmark of the jagged flash attention hot path on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one pass of the whole path -- forward, then backward (delta, dK/dV, dQ) -- over one seeded
synthetic batch already resident in HBM.  The default workload is the largest configuration
(c4_bimodal_bf16: B=512, H=8, D=128, 10 % of the samples 2048..4096 long, the rest 1..256).
Prints ONE JSON line:
  value           useful TFLOP/s of the whole step: (4 + 10) * H * D * sum L_b^2 flops / step time
                  (non-padded flops; the backward's recomputation of the scores is NOT counted)
  forward, backward
                  the same for the two calls on their own (us per call, useful TFLOP/s, % of bf16 MFMA peak)
  roofline        the kernel with the longest average launch, timed with HIP events on the launch
                  stream inside the timed region; kernels lists all of them
  cpu_baseline    the fp64 oracle timed on this host's cores on a bounded sample of the same workload
  all_configs     after the timed region: us per call (forward, forward + backward), useful TFLOP/s, % of peak and the
                  largest errors against the oracle for each of the five configurations
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # 256 CUs x 2.4 GHz x 4096 flop/clk/CU (dense bf16 MFMA)
# flops each kernel's definition requires per (query, key) pair, per head, per unit of D (2 per MAC):
#   forward: S and PV; dK/dV: S, dP, dV, dK; dQ: S, dP, dQ.  The delta / schedule kernels are bandwidth work.
KERNEL_GEMMS = {"fwd_bf16": 2, "fwd_bf16_dma": 2, "dkv_bf16": 4, "dq_bf16": 3, "dq_bf16_dma": 3, "dkv_bf16_dma": 4,
                "fwd_f32": 2}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_bimodal_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--forward-only", action="store_true", help="time the forward call alone (diagnostic)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the per-configuration block (timings and errors of all five)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (samples are independent and would shard with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.synthetic import make_workload

    binding.load()                                   # fails loudly if libjfa.so is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    t_gen = time.time()
    w = make_workload(args.workload, with_dout=True)
    assert w.dtype == "bf16", "the benchmark runs the bf16 path"
    t_gen = time.time() - t_gen

    def up(name):
        return torch.from_numpy(w.bits[name].view(np.int16)).view(torch.bfloat16).cuda()

    q, k, v, dout = up("q"), up("k"), up("v"), up("dout")
    offsets = torch.from_numpy(w.offsets).cuda()
    n, H, D = w.sum_B, w.H, w.D
    out = torch.empty_like(q)
    lse = torch.empty((H, n), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    delta = torch.empty((2, H, n), dtype=torch.float32, device="cuda")   # delta and the base-2 lse plane

    def forward():
        binding.jfa_forward(q, k, v, offsets, w.max_len, out=out, lse=lse)

    def backward():
        binding.jfa_backward(q, k, v, out, dout, lse, offsets, w.max_len, dq=dq, dk=dk, dv=dv, delta=delta)

    def step():
        forward()
        if not args.forward_only:
            backward()

    if args.calibrate_copy:
        # a plain elementwise copy of known size: 2^28 fp32 read + 2^28 fp32 written = 1 GiB each way
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, per-kernel HIP events recorded by the library on the launch stream ----
    binding.jfa_timing_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_kernel = binding.jfa_timing_read()
    binding.jfa_timing_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms_per_step_events = e0.elapsed_time(e1) / args.steps

    # ---- the two calls on their own (same buffers, after the timed region) ----
    def time_call(fn, reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    unit = H * D * float(w.S2)                       # flops of one GEMM = 2 * unit
    ms_fwd = time_call(forward, args.steps)
    ms_bwd = None if args.forward_only else time_call(backward, args.steps)

    def tf(flops, ms):
        return flops / (ms * 1e-3) / 1e12

    step_flops = 4 * unit if args.forward_only else 14 * unit
    value = tf(step_flops, ms_per_step)

    kernels = {}
    for name, (total_ms, launches) in per_kernel.items():
        avg_ms = total_ms / launches
        kk = {"avg_us": round(avg_ms * 1e3, 2), "launches": launches}
        if name in KERNEL_GEMMS:
            a = tf(2 * KERNEL_GEMMS[name] * unit, avg_ms)
            kk.update({"bound": "mfma", "achieved": round(a, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(a / PEAK_BF16_TFLOPS, 4)})
        kernels[name] = kk
    dom = max((kname for kname in kernels if "achieved" in kernels[kname]), key=lambda kname: kernels[kname]["avg_us"])
    roofline = {"kernel": dom, "bound": "mfma", "achieved": kernels[dom]["achieved"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": kernels[dom]["frac"], "avg_us": kernels[dom]["avg_us"],
                "traffic": recorded_traffic(w.name, dom)}

    result = {
        "metric": "jagged attention useful TFLOP/s (forward + backward step, non-padded flops only)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_hip_events": round(ms_per_step_events, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "pct_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "config": {"workload": w.name, "B": w.B, "H": H, "D": D, "max_len": w.max_len, "sum_B": n, "S2": w.S2,
                   "step": "forward" if args.forward_only else "forward+backward",
                   "useful_gflop_per_step": round(step_flops / 1e9, 1)},
        "forward": {"us_per_call": round(ms_fwd * 1e3, 1), "useful_tflops": round(tf(4 * unit, ms_fwd), 2),
                    "pct_bf16_mfma_peak": round(100 * tf(4 * unit, ms_fwd) / PEAK_BF16_TFLOPS, 2)},
        "roofline": roofline,
        "kernels": kernels,
        "workspace_bytes": binding.jfa_workspace_bytes(w.B, w.max_len, H, D, backward=True),
        "io_bytes": {"values_tensor": q.numel() * 2, "dense_padded_equivalent": w.B * w.max_len * H * D * 2},
        "input_generation_s": round(t_gen, 1),
    }
    if ms_bwd is not None:
        result["backward"] = {"us_per_call": round(ms_bwd * 1e3, 1), "useful_tflops": round(tf(10 * unit, ms_bwd), 2),
                              "pct_bf16_mfma_peak": round(100 * tf(10 * unit, ms_bwd) / PEAK_BF16_TFLOPS, 2)}
        result["forward_plus_backward_us"] = round((ms_fwd + ms_bwd) * 1e3, 1)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, args.forward_only)
    if not args.no_all_configs:
        del q, k, v, dout, out, lse, dq, dk, dv, delta
        torch.cuda.empty_cache()
        result["all_configs"] = all_configs(w)
    print(json.dumps(result), flush=True)


def all_configs(w_timed):
    """After the timed region: every one of the five configurations on its seeded inputs -- microseconds per call of
    the forward and of forward + backward (median of 3 timings of >= 20 ms each after 5 warm-up calls; a call is
    everything the entry point enqueues), useful TFLOP/s and % of the bf16 MFMA peak, cache-cold figures for the two
    whose tensors fit in the Infinity Cache (calls rotate over > 512 MB of copies), and the largest error against the
    oracle per tensor (max |gpu - oracle| and that over max |oracle|): whole tensors for c1 and c2, sampled
    (sample, head) pairs -- longest, shortest, median and random ones -- for the others."""
    import statistics

    import numpy as np
    import torch
    import oracle
    from paper_2409_15373_amd import binding
    from paper_2409_15373_amd.synthetic import CONFIGS, make_workload

    def timed_us(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / n

    def median_us(fn):
        for i in range(5):
            fn(i)
        torch.cuda.synchronize()
        n = max(3, int(20e3 / max(timed_us(fn, 3), 1e-3)) + 1)
        return statistics.median(timed_us(fn, n) for _ in range(3))

    res = {}
    for name in CONFIGS:
        w = w_timed if name == w_timed.name else make_workload(name, with_dout=True)
        is_bf16 = w.dtype == "bf16"
        H, D, n = w.H, w.D, w.sum_B

        def up(t):
            if is_bf16:
                return torch.from_numpy(w.bits[t].view(np.int16)).view(torch.bfloat16).cuda()
            return torch.from_numpy(getattr(w, t)).cuda()

        base = {t: up(t) for t in ("q", "k", "v", "dout")}
        footprint = 8 * base["q"].numel() * base["q"].element_size()
        copies = 1 if footprint >= 256e6 else int(512e6 // footprint) + 2
        x = {t: base[t].unsqueeze(0).repeat(copies, 1, 1, 1) for t in base}
        y = {t: torch.empty_like(x["q"]) for t in ("out", "dq", "dk", "dv")}
        planes = 2 if is_bf16 else 1
        stride = (planes * H * n + 63) // 64 * 64          # statistics blocks start on 256-byte boundaries
        lse_flat = torch.empty(copies * stride, device="cuda")
        st_flat = torch.empty(copies * stride, device="cuda")
        lse = [lse_flat[j * stride: j * stride + H * n].view(H, n) for j in range(copies)]
        stats = [st_flat[j * stride: j * stride + planes * H * n].view(planes, H, n) for j in range(copies)]
        off = torch.from_numpy(w.offsets).cuda()

        def fwd(i, m=1):
            j = i % m
            binding.jfa_forward(x["q"][j], x["k"][j], x["v"][j], off, w.max_len, out=y["out"][j], lse=lse[j])

        def step(i, m=1):
            j = i % m
            fwd(i, m)
            binding.jfa_backward(x["q"][j], x["k"][j], x["v"][j], y["out"][j], x["dout"][j], lse[j], off, w.max_len,
                                 dq=y["dq"][j], dk=y["dk"][j], dv=y["dv"][j], delta=stats[j])

        unit = H * D * float(w.S2)
        r = {"B": w.B, "H": H, "D": D, "max_len": w.max_len, "dtype": w.dtype, "sum_B": n, "S2": w.S2}
        for tag, fn, flops in (("fwd", fwd, 4 * unit), ("fwd_bwd", step, 14 * unit)):
            us = median_us(lambda i: fn(i, 1))
            r["us_" + tag] = round(us, 2)
            r["useful_tflops_" + tag] = round(flops / us / 1e6, 3)
            if is_bf16:
                r["pct_bf16_mfma_peak_" + tag] = round(100 * flops / us / 1e6 / PEAK_BF16_TFLOPS, 2)
            if copies > 1:
                r["us_" + tag + "_cache_cold"] = round(median_us(lambda i: fn(i, copies)), 2)
        # errors against the oracle on copy 0 (step(0) above left every output of that copy in place)
        step(0)
        torch.cuda.synchronize()
        if n * H <= 40000:
            pairs, rows, heads = None, slice(None), slice(None)
            r["error_sample"] = "whole tensors"
        else:
            order = np.argsort(w.lengths)
            rng = np.random.default_rng(3)
            picks = {(int(order[-1]), 0), (int(order[0]), H - 1), (int(order[len(order) // 2]), 1 % H)}
            while len(picks) < 12:
                picks.add((int(rng.integers(0, w.B)), int(rng.integers(0, H))))
            pairs = sorted(picks)
            rows = np.concatenate([np.arange(w.offsets[b], w.offsets[b + 1]) for b, _ in pairs])
            heads = np.concatenate([np.full(int(w.lengths[b]), h) for b, h in pairs])
            r["error_sample"] = f"{len(pairs)} (sample, head) pairs, lengths {int(min(w.lengths[b] for b, _ in pairs))}..{int(max(w.lengths[b] for b, _ in pairs))}"
        ref_out, ref_lse = oracle.forward(w.q, w.k, w.v, w.offsets, pairs=pairs)
        rdq, rdk, rdv, _ = oracle.backward(w.q, w.k, w.v, w.dout, w.offsets, pairs=pairs)
        g = lambda t: t.double().cpu().numpy()

        def err(got, ref, per_head_first=False):
            if pairs is None:
                a, b = got, ref
            elif per_head_first:
                a, b = got[heads, rows], ref[heads, rows]
            else:
                a, b = got[rows, heads], ref[rows, heads]
            e = float(np.abs(a - b).max())
            return {"max_abs_err": float(f"{e:.3e}"), "max_rel_err": float(f"{e / max(float(np.abs(b).max()), 1e-30):.3e}")}

        r["errors"] = {"out": err(g(y["out"][0]), ref_out), "lse": err(g(lse[0]), ref_lse, True),
                       "dq": err(g(y["dq"][0]), rdq), "dk": err(g(y["dk"][0]), rdk), "dv": err(g(y["dv"][0]), rdv)}
        res[name] = r
        print(f"[bench] {name}: fwd {r['us_fwd']} us, fwd+bwd {r['us_fwd_bwd']} us, out err {r['errors']['out']}", file=sys.stderr, flush=True)
        del x, y, base, lse, stats, lse_flat, st_flat
        torch.cuda.empty_cache()
    return res


def recorded_traffic(workload, kernel):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, copy-calibrated) of `kernel`, as recorded from the rocprofv3
    --pmc passes in profiles/<workload>_traffic.txt; None when no record exists for this kernel."""
    path = os.path.join(ROOT, "profiles", f"{workload}_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == kernel:
                return int(float(f[1]) + float(f[2]))
    except OSError:
        pass
    return None


def cpu_baseline(w, forward_only):
    """The oracle as it stands, on a bounded sample of (sample, head) pairs of the same workload."""
    import numpy as np
    import oracle
    oracle.build()
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    # sample: every `stride`-th sample in length order, one head each, trimmed to a pair budget of
    # about 2.5e10 score-matrix multiply-adds per core (roughly 10-30 s of oracle time)
    order = np.argsort(-w.lengths, kind="stable")
    budget = 2.5e10 * cores / (w.D * (2 if forward_only else 7))
    pairs, used = [], 0.0
    stride = max(1, w.B // 64)
    for idx, b in enumerate(order[::stride]):
        cost = float(w.lengths[b]) ** 2
        if used + cost > budget and pairs:
            continue
        pairs.append((int(b), idx % w.H))
        used += cost
    t0 = time.perf_counter()
    _, _, threads = oracle.forward(w.q, w.k, w.v, w.offsets, pairs=pairs, return_threads=True)
    if not forward_only:
        oracle.backward(w.q, w.k, w.v, w.dout, w.offsets, pairs=pairs)
    dt = time.perf_counter() - t0
    flops = (4 if forward_only else 14) * w.D * used
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": f"{len(pairs)} (sample, head) pairs of {w.name} (every {stride}-th sample by length, "
                      f"lengths {int(min(w.lengths[b] for b, _ in pairs))}..{int(max(w.lengths[b] for b, _ in pairs))}, "
                      f"{used:.3g} query-key pairs), fp64, "
                      + ("forward" if forward_only else "forward+backward")}


if __name__ == "__main__":
    main()
