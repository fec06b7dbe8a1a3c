#!/usr/bin/env python3
"""Benchmark of the PruneTrain conv-layer hot path on one MI355X.

One *step* = one pass of the whole hot path over one batch of synthetic input:
  (1) training step at full width   - the 53 ResNet-50 convolutions at batch 64 (224x224 image):
      group norms of every layer (+ bf16 shadow weights), conv_fwd per layer, conv_bwd_data and
      conv_bwd_weight per layer in reverse order, group-lasso gradient added to every dW;
  (2) reconfiguration sweep         - group_norms + zero_groups on every layer, reconcile + plan on
      every channel edge, then compaction of weights, momentum, normalisation vectors and the saved
      input activations (a fraction of each edge's channels zeroed on the pruned-width model);
  (3) training step at pruned width - the same 53 layers at ragged widths (keep fractions U[0.4,0.9]).
`value` = convolution FLOPs of (1)+(3) divided by the time of the whole step, inputs resident in HBM.
The launch sequences are captured once into HIP graphs and replayed (the survivor counts the sweep
reads back are checked on every step).  Prints ONE JSON line on stdout; --detail FILE also writes
per-layer tables to FILE.
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


def cpu_baseline(max_seconds: float = 25.0, batch: int = 16):
    """The fp64 oracle, as it stands, on the host cores: fwd + bwd_data + bwd_weight of the full-width
    ResNet-50 layer shapes at a reduced batch, stopping after ~max_seconds."""
    import oracle
    from paper_1901_09290_amd import workloads as wl
    layers, _ = wl.resnet50_layers(N=batch)
    rng = np.random.Generator(np.random.PCG64(2))
    flops, secs, done = 0, 0.0, 0
    shapes = wl.distinct_shapes(layers)
    for spec, _cnt in shapes:
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
    return {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 nested-loop oracle, fwd+bwd_data+bwd_weight of the first {done} of {len(shapes)} distinct "
                      f"ResNet-50 layer shapes at batch {batch} ({flops / 1e9:.1f} GFLOP in {secs:.1f} s)"}


def conv_bytes(spec, which: str) -> int:
    """Algorithmic HBM bytes of one convolution pass (bf16 activations and weights, fp32 dw)."""
    st2 = spec.stride * spec.stride if spec.R == 1 else 1      # a strided 1x1 touches 1/stride^2 of its input pixels
    x = 2 * spec.N * spec.H * spec.W * spec.C // st2
    y = 2 * spec.N * spec.P * spec.Q * spec.K
    w = 2 * spec.params
    if which == "bwd_weight":
        return x + y + 4 * spec.params
    return x + y + w


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--sparsity", type=float, default=0.3, help="fraction of each edge zeroed in the sweep")
    ap.add_argument("--detail", metavar="FILE", default=None, help="also write per-layer tables to FILE")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the weight gradients on the same stream as the input-gradient chain")
    ap.add_argument("--no-fused-lasso", action="store_true",
                    help="add the regulariser's gradient in a pass of its own after the weight gradients")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="only the timed step and its phases (no per-family timings)")
    ap.add_argument("--wgrad-streams", type=int, default=None, help="side streams the weight gradients alternate between")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a plain elementwise kernel of known size (reads 1 GiB, writes 1 GiB): the "
                         "reference against which hardware byte counters of a profiler run are scaled")
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
    if args.wgrad_streams is not None:
        hz.WGRAD_STREAMS = args.wgrad_streams
    torch.cuda.set_device(0)
    N = args.batch

    # ---- synthetic workloads ------------------------------------------------------------------ #
    full_specs, edges = wl.resnet50_layers(N=N)
    keep = wl.pruned_keep_sets(edges, seed=3)
    pruned_specs, pruned_edges = wl.with_widths(full_specs, edges, [k.size for k in keep])
    full = hz.Network(hz.build_network(full_specs, seed=2))
    pruned = hz.Network(hz.build_network(pruned_specs, seed=3))
    full.overlap_wgrad = pruned.overlap_wgrad = not args.no_overlap
    full.fuse_lasso = pruned.fuse_lasso = not args.no_fused_lasso
    rng = np.random.Generator(np.random.PCG64(10 + int(round(args.sparsity * 10))))
    zero_sets = wl.zeroed_channel_sets(pruned_edges, args.sparsity, rng)
    rweights = wl.network_weights(pruned_specs, pruned_edges, zero_sets, rng)
    rmodel = hz.ReconfigModel(pruned_specs, pruned_edges, rweights, seed=11)
    torch.cuda.synchronize()
    f_full, f_pruned = full.step_flops, pruned.step_flops
    log(f"full: {f_full / 1e12:.3f} TFLOP/step, pruned: {f_pruned / 1e12:.3f} TFLOP/step, "
        f"mem {torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    # ---- eager warm-up (also the first launches that set kernel attributes) ---------------------- #
    for _ in range(max(1, args.warmup)):
        full.train_step(LAMBDA)
        rmodel.sweep(THRESHOLD)
        pruned.train_step(LAMBDA)
    torch.cuda.synchronize()
    counts0 = rmodel.new_counts.copy()
    expect = np.array([e.n - z.size for e, z in zip(pruned_edges, zero_sets)])
    assert np.array_equal(counts0, expect), "survivor counts differ from the zero pattern that was planted"

    use_graph = not args.no_graph
    if use_graph:
        side = torch.cuda.Stream()
        g1, g2 = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g1, stream=side):
                full.train_step(LAMBDA)
                rmodel.detect(THRESHOLD)
            with torch.cuda.graph(g2, stream=side):
                rmodel.compact(counts0)
                pruned.train_step(LAMBDA)
        torch.cuda.synchronize()

        def step():
            g1.replay()
            cnt = rmodel.counts.cpu().numpy()          # the sweep's one synchronising read-back
            if not np.array_equal(cnt, counts0):
                raise RuntimeError("survivor counts changed between steps")
            g2.replay()
    else:
        def step():
            full.train_step(LAMBDA)
            rmodel.sweep(THRESHOLD)
            pruned.train_step(LAMBDA)

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

    # ---- per-phase and per-family timing (same launches, HIP events on the launch stream) -------- #
    def timed(fn, reps):
        fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    reps = max(3, min(10, args.steps))
    if use_graph:
        gf, gp, gd, gc = (torch.cuda.CUDAGraph() for _ in range(4))
        with torch.cuda.stream(side):
            with torch.cuda.graph(gf, stream=side):
                full.train_step(LAMBDA)
            with torch.cuda.graph(gp, stream=side):
                pruned.train_step(LAMBDA)
            with torch.cuda.graph(gd, stream=side):
                rmodel.detect(THRESHOLD)
            with torch.cuda.graph(gc, stream=side):
                rmodel.compact(counts0)
        torch.cuda.synchronize()
        t_full, t_pruned = timed(gf.replay, reps), timed(gp.replay, reps)
        t_detect, t_compact = timed(gd.replay, reps), timed(gc.replay, reps)
    else:
        t_full = timed(lambda: full.train_step(LAMBDA), reps)
        t_pruned = timed(lambda: pruned.train_step(LAMBDA), reps)
        t_detect = timed(lambda: rmodel.detect(THRESHOLD), reps)
        t_compact = timed(lambda: rmodel.compact(counts0), reps)

    if args.quick:
        print(json.dumps({"value": round(value, 3), "ms_per_step": round(ms_step, 4), "full_ms": round(t_full, 4),
                          "pruned_ms": round(t_pruned, 4), "detect_ms": round(t_detect, 4),
                          "compact_ms": round(t_compact, 4), "wgrad_streams": hz.WGRAD_STREAMS}), flush=True)
        return

    # kernel families: every layer's call of one kind back to back between two events
    fam = {}
    for tag, net in (("full", full), ("pruned", pruned)):
        L = net.layers
        fam[tag] = {
            "fwd": timed(lambda: [l.fwd(net.ws) for l in L], 3),
            "bwd_data": timed(lambda: [l.bwd_data_crsk() for l in L], 3),
            "bwd_weight": timed(lambda: [l.bwd_weight(net.ws) for l in L], 3),
            "bwd_weight_lasso": timed(lambda: [l.bwd_weight_lasso(net.ws, LAMBDA) for l in L], 3),
            "group_norms": timed(lambda: B.group_norms_batched(net.norm_jobs, net.ws_norms), 5),
            "group_lasso_grad": timed(lambda: B.group_lasso_grad_batched(net.lasso_jobs, LAMBDA), 5),
            # not part of the timed step: the optimizer step with the regulariser folded in (lr = 0: weights unchanged)
            "optimizer_step_fused": timed(lambda: net.optimizer_step(LAMBDA, 0.0, 0.9, 1e-4), 5),
            # not part of the timed step either: feature normalisation of every convolution output, forward and backward
            "fwd+bn": timed(lambda: net.fwd_bn_all(False), 3),
            "fwd+bn_fused": timed(lambda: net.fwd_bn_all(True), 3),
            "bn_fwd": timed(net.bn_fwd_all, 3),
            "bn_bwd": timed(net.bn_bwd_all, 3),
        }
    fl = {tag: {"fwd": sum(l.spec.flops for l in net.layers),
                "bwd_data": sum(l.spec.flops for l in net.layers if l.dx is not None),
                "bwd_weight": sum(l.spec.flops for l in net.layers)} for tag, net in (("full", full), ("pruned", pruned))}
    by = {tag: {k: sum(conv_bytes(l.spec, k) for l in net.layers if not (k == "bwd_data" and l.dx is None))
                for k in ("fwd", "bwd_data", "bwd_weight")} for tag, net in (("full", full), ("pruned", pruned))}
    params = {tag: sum(l.spec.params for l in net.layers) for tag, net in (("full", full), ("pruned", pruned))}

    # dominant kernel of the step: k_igemm_dl serves conv_fwd and conv_bwd_data, k_wgrad_dl (+ k_wgrad_reduce)
    # conv_bwd_weight; the one with the larger time over both widths is reported against its roof
    nets = (full, pruned)
    tot = {k: fam["full"][k] + fam["pruned"][k] for k in ("fwd", "bwd_data", "bwd_weight")}
    kernels = {"k_igemm_dl (conv_fwd + conv_bwd_data launches)": ("fwd", "bwd_data"),
               "k_wgrad_dl + k_wgrad_reduce (conv_bwd_weight launches)": ("bwd_weight",)}
    dom_kernel = max(kernels, key=lambda k: sum(tot[f] for f in kernels[k]))
    fams = kernels[dom_kernel]

    def has(l, f):
        return not (f == "bwd_data" and l.dx is None)

    def launches(l, f):  # the input gradient is one launch per stride-parity class that holds a filter tap
        s = l.spec
        return min(s.stride, s.R) * min(s.stride, s.S) if f == "bwd_data" else 1
    n_launch = sum(launches(l, f) for f in fams for net in nets for l in net.layers if has(l, f))
    dom_flops = sum(fl[t][f] for f in fams for t in ("full", "pruned"))
    dom_bytes = sum(by[t][f] for f in fams for t in ("full", "pruned"))
    dom_s = sum(tot[f] for f in fams) * 1e-3
    # which roof bounds this kernel on this workload: time at the HBM peak vs time at the bf16 MFMA peak
    t_hbm, t_mfma = dom_bytes / (PEAK_HBM_GBS * 1e9), dom_flops / (PEAK_BF16_TFLOPS * 1e12)
    # per-layer roof: a layer cannot finish before max(its bytes at the HBM peak, its flops at the MFMA peak)
    t_roof = sum(max(conv_bytes(l.spec, f) / (PEAK_HBM_GBS * 1e9), l.spec.flops / (PEAK_BF16_TFLOPS * 1e12))
                 for f in fams for net in nets for l in net.layers if has(l, f))
    if t_hbm >= t_mfma:
        ach, peak, unit, bound = dom_bytes / dom_s / 1e9, PEAK_HBM_GBS, "GB/s", "hbm"
    else:
        ach, peak, unit, bound = dom_flops / dom_s / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s", "mfma"
    roofline = {"bound": bound, "kernel": dom_kernel, "achieved": round(ach, 2), "peak": peak, "unit": unit,
                "frac": round(ach / peak, 4), "traffic": None,
                "avg_launch_ms": round(dom_s * 1e3 / n_launch, 5), "launches_per_step": n_launch,
                "bytes_per_launch": dom_bytes / n_launch, "flops_per_launch": dom_flops / n_launch,
                "tflops": round(dom_flops / dom_s / 1e12, 2), "frac_mfma_peak": round(dom_flops / dom_s / 1e12 / PEAK_BF16_TFLOPS, 4),
                "frac_of_per_layer_roof": round(t_roof / dom_s, 4)}

    # HBM traffic of the dominant kernel, measured separately with hardware counters (this file is written from
    # two `rocprofv3 --pmc` runs of this script; see its header for the commands and the scale factors)
    tpath = os.path.join(ROOT, "profiles", "bench_resnet50_b64_hbm_traffic.txt")
    if os.path.exists(tpath):
        import re
        pat = (r"per k_igemm_dl launch .*?= ([0-9.]+) MB of HBM traffic" if "k_igemm_dl" in dom_kernel
               else r"per pt_conv_bwd_weight call .*?= ([0-9.]+) MB of HBM traffic")
        m = re.search(pat, open(tpath).read())
        if m:
            roofline["traffic"] = float(m.group(1)) * 1e6
            roofline["traffic_unit"] = "bytes per launch (FETCH_SIZE x 2.0 + WRITE_SIZE, from profiles/)"

    ab = rmodel.algorithmic_bytes()
    sweep_bytes = sum(ab.values())
    t_sweep = t_detect + t_compact

    def fam_table(tag):
        out = {}
        for k in ("fwd", "bwd_data", "bwd_weight"):
            t = fam[tag][k]
            out[k] = {"ms": round(t, 4), "tflops": round(fl[tag][k] / (t * 1e-3) / 1e12, 1),
                      "algorithmic_GBps": round(by[tag][k] / (t * 1e-3) / 1e9, 1)}
        # what the step launches when the regulariser's gradient is folded into the weight gradient (the default)
        out["bwd_weight_with_lasso"] = {"ms": round(fam[tag]["bwd_weight_lasso"], 4)}
        tn, tl = fam[tag]["group_norms"], fam[tag]["group_lasso_grad"]
        out["group_norms"] = {"ms": round(tn, 4), "GBps": round(6 * params[tag] / (tn * 1e-3) / 1e9, 1),
                              "frac_hbm_peak": round(6 * params[tag] / (tn * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        out["group_lasso_grad(separate pass)"] = {"ms": round(tl, 4), "GBps": round(12 * params[tag] / (tl * 1e-3) / 1e9, 1),
                                   "frac_hbm_peak": round(12 * params[tag] / (tl * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        to = fam[tag]["optimizer_step_fused"]
        out["optimizer_step_fused(not in step)"] = {"ms": round(to, 4), "GBps": round(20 * params[tag] / (to * 1e-3) / 1e9, 1),
                                                    "frac_hbm_peak": round(20 * params[tag] / (to * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        out["fwd+bn(not in step)"] = {"separate_ms": round(fam[tag]["fwd+bn"], 4),
                                      "statistics_in_conv_epilogue_ms": round(fam[tag]["fwd+bn_fused"], 4)}
        for k, bpe in (("bn_fwd", 6), ("bn_bwd", 10)):
            t = fam[tag][k]
            out[k + "(not in step)"] = {"ms": round(t, 4), "GBps": round(bpe * net_of[tag].bn_elements / (t * 1e-3) / 1e9, 1),
                                        "frac_hbm_peak": round(bpe * net_of[tag].bn_elements / (t * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        return out

    net_of = {"full": full, "pruned": pruned}
    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-50 conv layers (53), batch {N}, 224x224, NHWC bf16: train step at full width "
                               f"(cfg3) + reconfiguration sweep at {int(args.sparsity * 100)}% zeroed groups (cfg5) + "
                               "train step at ragged pruned widths (cfg4)",
                   "lambda": LAMBDA, "threshold": THRESHOLD, "hip_graphs": use_graph,
                   "wgrad_side_streams": 0 if args.no_overlap else hz.WGRAD_STREAMS,
                   "lasso_in_wgrad_reduce": bool(full.fuse_lasso and full.overlap_wgrad)},
        "roofline": roofline,
        "breakdown": {
            "wall_ms_per_step": round(wall_ms, 4),
            "full_width": {"ms": round(t_full, 4), "tflops": round(f_full / (t_full * 1e-3) / 1e12, 2),
                           "frac_mfma_peak": round(f_full / (t_full * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
            "pruned_width": {"ms": round(t_pruned, 4), "tflops": round(f_pruned / (t_pruned * 1e-3) / 1e12, 2),
                             "frac_mfma_peak": round(f_pruned / (t_pruned * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                             "flop_ratio_vs_full": round(f_pruned / f_full, 4),
                             "time_ratio_vs_full": round(t_pruned / t_full, 4)},
            "kernel_families_full": fam_table("full"),
            "kernel_families_pruned": fam_table("pruned"),
            "reconfig_sweep": {"ms": round(t_sweep, 4), "detect_ms": round(t_detect, 4), "compact_ms": round(t_compact, 4),
                               "algorithmic_MB": {k: round(v / 1e6, 1) for k, v in ab.items()},
                               "GBps": round(sweep_bytes / (t_sweep * 1e-3) / 1e9, 1),
                               "frac_hbm_peak": round(sweep_bytes / (t_sweep * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        },
    }
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.neg(src, out=dst)       # one launch: 2^30 bytes read, 2^30 bytes written
        torch.cuda.synchronize()
        out["copy_probe"] = {"kernel": "torch.neg (vectorized elementwise)", "read_bytes": 1 << 30, "write_bytes": 1 << 30}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()

    if args.detail:
        calls = ("fwd", "bwd_data", "bwd_weight")
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            for tag, net in (("full", full), ("pruned", pruned)):
                f.write(f"== {tag} ==  per call, eager (includes launch latency): us, TFLOP/s, algorithmic GB/s\n")
                for l in net.layers:
                    row = f"{l.spec.name:18s} {str(l.spec.shape_key()):36s} {l.spec.flops / 1e9:7.2f} GF |"
                    for c in calls:
                        if c == "bwd_data" and l.dx is None:
                            row += f" {'-':>8s} {'':>5s} {'':>5s} |"
                            continue
                        t = timed((lambda l=l: l.bwd_data_crsk()) if c == "bwd_data" else
                                  (lambda l=l, c=c: getattr(l, c)(net.ws)), 3)
                        row += (f" {t * 1e3:8.1f} {l.spec.flops / (t * 1e-3) / 1e12:5.0f} "
                                f"{conv_bytes(l.spec, c) / (t * 1e-3) / 1e9:5.0f} |")
                    f.write(row + "\n")
            f.write(json.dumps(out, indent=1) + "\n")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
