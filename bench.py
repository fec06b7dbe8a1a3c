#!/usr/bin/env python3
"""Benchmark of the PruneTrain conv-layer hot path on one MI355X.

One *step* = one pass of the whole hot path over one batch of synthetic input:
  (1) training step at full width   - the 53 ResNet-50 convolutions at batch 64 (224x224 image):
      per layer group_norms(+bf16 shadow), conv_fwd, conv_bwd_data, conv_bwd_weight, group_lasso_grad;
  (2) reconfiguration sweep         - group_norms + zero_groups on every layer, reconcile + plan on
      every channel edge, then compaction of weights, momentum, normalisation vectors and the saved
      input activations (30 % of each edge's channels zeroed on the pruned-width model);
  (3) training step at pruned width - the same 53 layers at ragged widths (keep fractions U[0.4,0.9]).
`value` = convolution FLOPs of (1)+(3) divided by the time of the whole step, inputs resident in HBM.

Prints ONE JSON line on stdout.  --detail writes a per-layer table to gpurun_out/.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "conv train-step TFLOP/s (fwd+bwd) at full vs pruned widths; %MFMA & %HBM peak"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
LAMBDA = 1e-3
THRESHOLD = 1e-6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(max_seconds: float = 30.0):
    """The fp64 oracle, as it stands, on the host cores: fwd + bwd_data + bwd_weight of the full-width
    ResNet-50 layer shapes at batch 1 (1/64 of the workload's batch), stopping after ~max_seconds."""
    import oracle
    from paper_1901_09290_amd import workloads as wl
    layers, _ = wl.resnet50_layers(N=1)
    rng = np.random.Generator(np.random.PCG64(2))
    flops, secs, done = 0, 0.0, 0
    for spec, _cnt in wl.distinct_shapes(layers):
        t = wl.conv_tensors(spec, rng)
        s = oracle.shape_of(spec)
        t0 = time.perf_counter()
        oracle.conv_fwd(s, t["x"], t["w"])
        if not spec.first:
            oracle.conv_bwd_data(s, t["dy"], t["w"])
        oracle.conv_bwd_weight(s, t["x"], t["dy"])
        secs += time.perf_counter() - t0
        flops += spec.flops * (2 if spec.first else 3)
        done += 1
        if secs > max_seconds:
            break
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 nested-loop oracle, fwd+bwd_data+bwd_weight of the first {done} distinct ResNet-50 "
                      f"layer shapes at batch 1 ({flops / 1e9:.1f} GFLOP in {secs:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--sparsity", type=float, default=0.3, help="fraction of each edge zeroed in the sweep")
    ap.add_argument("--detail", action="store_true", help="write a per-layer table under gpurun_out/")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1901_09290_amd import binding as B
    from paper_1901_09290_amd import harness as hz
    from paper_1901_09290_amd import workloads as wl

    B.lib()  # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    N = args.batch

    # ---- synthetic workloads ------------------------------------------------------------------ #
    full_specs, edges = wl.resnet50_layers(N=N)
    keep = wl.pruned_keep_sets(edges, seed=3)
    pruned_specs, pruned_edges = wl.with_widths(full_specs, edges, [k.size for k in keep])
    full = hz.build_network(full_specs, seed=2)
    pruned = hz.build_network(pruned_specs, seed=3)
    ws = hz.make_workspace(full + pruned)
    rng = np.random.Generator(np.random.PCG64(10 + int(round(args.sparsity * 10))))
    zero_sets = wl.zeroed_channel_sets(pruned_edges, args.sparsity, rng)
    rweights = wl.network_weights(pruned_specs, pruned_edges, zero_sets, rng)
    rmodel = hz.ReconfigModel(pruned_specs, pruned_edges, rweights, seed=11)
    torch.cuda.synchronize()
    f_full = sum(l.step_flops for l in full)
    f_pruned = sum(l.step_flops for l in pruned)
    log(f"full: {f_full / 1e12:.3f} TFLOP/step, pruned: {f_pruned / 1e12:.3f} TFLOP/step, "
        f"mem {torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    def step():
        hz.train_step(full, ws, LAMBDA)
        rmodel.sweep(THRESHOLD)
        hz.train_step(pruned, ws, LAMBDA)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps -------------------------------------------------------- #
    ev = lambda: torch.cuda.Event(enable_timing=True)
    e0, e1 = ev(), ev()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_step = e0.elapsed_time(e1) / args.steps
    value = (f_full + f_pruned) / (ms_step * 1e-3) / 1e12

    # ---- per-phase and per-call timing (same launches, HIP events on the launch stream) -------- #
    def timed(fn, reps):
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    reps = max(1, args.steps)
    t_full = timed(lambda: hz.train_step(full, ws, LAMBDA), reps)
    t_pruned = timed(lambda: hz.train_step(pruned, ws, LAMBDA), reps)
    t_sweep = timed(lambda: rmodel.sweep(THRESHOLD), reps)
    t_detect = timed(lambda: rmodel.detect(THRESHOLD), reps)

    calls = ("norms", "fwd", "bwd_data", "bwd_weight", "lasso")
    per = {}
    for tag, net in (("full", full), ("pruned", pruned)):
        rows = []
        for l in net:
            r = {"name": l.spec.name, "shape": list(l.spec.shape_key()), "flops": l.spec.flops}
            for c in calls:
                fn = (lambda l=l, c=c: l.lasso(LAMBDA)) if c == "lasso" else (lambda l=l, c=c: getattr(l, c)(ws))
                if c == "bwd_data" and l.dx is None:
                    r[c] = 0.0
                    continue
                r[c] = timed(fn, 3)
            rows.append(r)
        per[tag] = rows

    def conv_rate(rows, key, skip_first=False):
        f = sum(r["flops"] for r in rows if not (skip_first and r[key] == 0.0))
        t = sum(r[key] for r in rows)
        return f / (t * 1e-3) / 1e12 if t > 0 else 0.0, t

    # dominant kernel: the implicit-GEMM forward/input-gradient kernel (fwd + bwd_data launches)
    ig_f = sum(r["flops"] * (1 + (r["bwd_data"] > 0)) for tag in per for r in per[tag])
    ig_t = sum(r["fwd"] + r["bwd_data"] for tag in per for r in per[tag])
    ig_launches = sum(1 + (r["bwd_data"] > 0) for tag in per for r in per[tag])
    ig_rate = ig_f / (ig_t * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "k_igemm (conv_fwd + conv_bwd_data launches of one step)",
                "achieved": round(ig_rate, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ig_rate / PEAK_BF16_TFLOPS, 4), "traffic": None,
                "avg_launch_ms": round(ig_t / ig_launches, 5), "flops_per_launch": ig_f / ig_launches}

    ab = rmodel.algorithmic_bytes()
    sweep_bytes = sum(ab.values())
    norms_bytes_full = sum(4 * l.spec.params + 2 * l.spec.params for l in full)     # read fp32, write bf16 shadow
    norms_t_full = sum(r["norms"] for r in per["full"])
    lasso_bytes_full = sum(12 * l.spec.params for l in full)
    lasso_t_full = sum(r["lasso"] for r in per["full"])

    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-50 conv layers (53), batch {N}, 224x224, NHWC bf16: train step at full width "
                               f"(cfg3) + reconfiguration sweep at {int(args.sparsity * 100)}% zeroed groups (cfg5) + "
                               "train step at ragged pruned widths (cfg4)",
                   "lambda": LAMBDA, "threshold": THRESHOLD},
        "roofline": roofline,
        "breakdown": {
            "wall_ms_per_step": round(wall_ms, 4),
            "full_width": {"ms": round(t_full, 4), "tflops": round(f_full / (t_full * 1e-3) / 1e12, 2),
                           "frac_mfma_peak": round(f_full / (t_full * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
            "pruned_width": {"ms": round(t_pruned, 4), "tflops": round(f_pruned / (t_pruned * 1e-3) / 1e12, 2),
                             "frac_mfma_peak": round(f_pruned / (t_pruned * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                             "flop_ratio_vs_full": round(f_pruned / f_full, 4),
                             "time_ratio_vs_full": round(t_pruned / t_full, 4)},
            "conv_tflops_full": {c: round(conv_rate(per["full"], c)[0], 2) for c in ("fwd", "bwd_data", "bwd_weight")},
            "conv_tflops_pruned": {c: round(conv_rate(per["pruned"], c)[0], 2)
                                   for c in ("fwd", "bwd_data", "bwd_weight")},
            "reconfig_sweep": {"ms": round(t_sweep, 4), "detect_ms": round(t_detect, 4),
                               "algorithmic_MB": round(sweep_bytes / 1e6, 1),
                               "GBps": round(sweep_bytes / (t_sweep * 1e-3) / 1e9, 1),
                               "frac_hbm_peak": round(sweep_bytes / (t_sweep * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
            "group_norms_full": {"ms": round(norms_t_full, 4),
                                 "GBps": round(norms_bytes_full / (norms_t_full * 1e-3) / 1e9, 1)},
            "group_lasso_grad_full": {"ms": round(lasso_t_full, 4),
                                      "GBps": round(lasso_bytes_full / (lasso_t_full * 1e-3) / 1e9, 1)},
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()

    if args.detail:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_detail.txt"), "w") as f:
            for tag in per:
                f.write(f"== {tag} ==  (ms, TFLOP/s per call)\n")
                f.write(f"{'layer':22s} {'N,H,W,C,K,R,S,st,pad':34s} {'GF':>7s} | {'norms':>7s} {'fwd':>7s} {'TF/s':>6s} "
                        f"{'bwd_d':>7s} {'TF/s':>6s} {'bwd_w':>7s} {'TF/s':>6s} {'lasso':>7s}\n")
                for r in per[tag]:
                    tf = lambda k: (r["flops"] / (r[k] * 1e-3) / 1e12) if r[k] > 0 else 0.0
                    f.write(f"{r['name']:22s} {str(tuple(r['shape'])):34s} {r['flops'] / 1e9:7.2f} | {r['norms']:7.4f} "
                            f"{r['fwd']:7.4f} {tf('fwd'):6.0f} {r['bwd_data']:7.4f} {tf('bwd_data'):6.0f} "
                            f"{r['bwd_weight']:7.4f} {tf('bwd_weight'):6.0f} {r['lasso']:7.4f}\n")
            f.write(json.dumps(out, indent=1) + "\n")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
