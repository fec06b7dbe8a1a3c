#!/usr/bin/env python3
"""Benchmark of the PruneTrain conv-layer hot path on one MI355X.

One *step* = one pass of the whole hot path over one batch of synthetic input:
  (1) training step at full width   - the 53 ResNet-50 convolutions at batch 64 (224x224 image):
      group norms of every layer (+ bf16 shadow weights), conv_fwd per layer, conv_bwd_data and
      conv_bwd_weight per layer in reverse order, group-lasso gradient added to every dW;
  (2) reconfiguration sweep         - group norms + zero masks of every layer, reconcile + plan on
      every channel edge, then compaction of weights, momentum, normalisation vectors and the saved
      input activations (a fraction of each edge's channels zeroed on the pruned-width model);
  (3) training step at pruned width - the same 53 layers at ragged widths (keep fractions U[0.4,0.9]).
`value` = convolution FLOPs of (1)+(3) divided by the time of the whole step, inputs resident in HBM.
The launch sequences are captured once into HIP graphs and replayed (the survivor counts the sweep
reads back are checked on every step).  Prints ONE JSON line on stdout.

Every figure besides `value` is a median over --reps timed repetitions (HIP events on the stream
the kernels are launched on): the phases of the step, and every kernel family as one graph holding
each layer's call of that kind back to back.  Each family is graded against the sum of its layers'
own roofs, max(bytes / HBM peak, FLOPs / MFMA peak), per width.

--layer-pass FILE runs no timed step: it launches every layer's calls one by one, eagerly, with a
marker kernel between calls, and writes the list of calls to FILE.  Run under a kernel trace or a
counter collection, that is the input of paper_1901_09290_amd/profile_report.py.
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
CONV_KINDS = ("fwd", "bwd_data", "bwd_weight")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# --------------------------------------------------------------------------------------------- #
# algorithmic work
# --------------------------------------------------------------------------------------------- #
def conv_bytes(spec, which: str) -> int:
    """Algorithmic HBM bytes of one convolution pass (bf16 activations and weights, fp32 dw)."""
    st2 = spec.stride * spec.stride if spec.R == 1 else 1      # a strided 1x1 touches 1/stride^2 of its input pixels
    x = 2 * spec.N * spec.H * spec.W * spec.C // st2
    y = 2 * spec.N * spec.P * spec.Q * spec.K
    w = 2 * spec.params
    if which.startswith("bwd_weight"):
        return x + y + 4 * spec.params
    return x + y + w


def conv_roof_s(spec, which: str) -> float:
    """A layer cannot finish before max(its bytes at the HBM peak, its FLOPs at the bf16 MFMA peak)."""
    return max(conv_bytes(spec, which) / (PEAK_HBM_GBS * 1e9), spec.flops / (PEAK_BF16_TFLOPS * 1e12))


def has_call(spec, which: str) -> bool:
    return not (which == "bwd_data" and spec.first)


# --------------------------------------------------------------------------------------------- #
# the oracle on the host cores
# --------------------------------------------------------------------------------------------- #
def _oracle_convs(wl, oracle, batch: int, max_seconds: float):
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
    return flops, secs, done, len(shapes)


def cpu_baseline(sparsity: float):
    """The fp64 oracle, as it stands, on the host cores.  `value`: fwd + bwd_data + bwd_weight of the full-width
    ResNet-50 layer shapes at a reduced batch on all cores, in the unit of the metric.  Beside it the same on one
    thread, and the bandwidth-bound steps (group norms, regulariser gradient, weight and activation compaction) on
    layers of the pruned-width model, in GB/s of the bytes the GPU path is charged for the same step."""
    import oracle
    from paper_1901_09290_amd import workloads as wl
    cores = oracle.num_threads()
    flops, secs, done, n_shapes = _oracle_convs(wl, oracle, 16, 12.0)
    oracle.set_num_threads(1)
    f1, s1, d1, _ = _oracle_convs(wl, oracle, 2, 6.0)
    oracle.set_num_threads(cores)

    # bandwidth-bound steps on the pruned-width model's layers (weights of all 53 layers, activations at batch 2)
    full_specs, edges = wl.resnet50_layers(N=2)
    keep = wl.pruned_keep_sets(edges, seed=3)
    specs, pedges = wl.with_widths(full_specs, edges, [k.size for k in keep])
    rng = np.random.Generator(np.random.PCG64(10 + int(round(sparsity * 10))))
    zero_sets = wl.zeroed_channel_sets(pedges, sparsity, rng)
    weights = [w.astype(np.float64) for w in wl.network_weights(specs, pedges, zero_sets, rng)]
    keep_idx = [np.setdiff1d(np.arange(e.n, dtype=np.int32), z).astype(np.int32) for e, z in zip(pedges, zero_sets)]
    hb = {}
    for threads in (cores, 1):
        oracle.set_num_threads(threads)
        t_n = t_l = t_w = t_a = 0.0
        b_n = b_l = b_w = b_a = 0
        for s, w in zip(specs, weights):
            t0 = time.perf_counter()
            on, inn = oracle.group_norms(w)
            t_n += time.perf_counter() - t0
            b_n += 4 * s.params
            dw = np.zeros_like(w)
            t0 = time.perf_counter()
            oracle.group_lasso_grad(w, on, inn, LAMBDA, 1 if s.first else 3, dw)
            t_l += time.perf_counter() - t0
            b_l += 12 * s.params
            ik = keep_idx[s.out_edge] if s.out_edge is not None else None
            ic = keep_idx[s.in_edge] if s.in_edge is not None else None
            t0 = time.perf_counter()
            wc = oracle.compact_weights(w, ik, ic)
            t_w += time.perf_counter() - t0
            b_w += 2 * 4 * wc.size
        for s in specs[1:12]:
            ic = keep_idx[s.in_edge]
            x = wl.bf16_bits(wl.to_bf16_grid(rng.standard_normal((s.N, s.H, s.W, s.C), dtype=np.float32)))
            t0 = time.perf_counter()
            oracle.compact_nhwc(x, ic)
            t_a += time.perf_counter() - t0
            b_a += 2 * 2 * s.N * s.H * s.W * ic.size
        hb["all_cores" if threads == cores else "one_thread"] = {
            "group_norms_GBps": round(b_n / t_n / 1e9, 3), "group_lasso_grad_GBps": round(b_l / t_l / 1e9, 3),
            "compact_weights_GBps": round(b_w / t_w / 1e9, 3), "compact_nhwc_GBps": round(b_a / t_a / 1e9, 3)}
    oracle.set_num_threads(cores)
    return {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 nested-loop oracle, fwd+bwd_data+bwd_weight of the first {done} of {n_shapes} distinct "
                      f"ResNet-50 layer shapes at batch 16 ({flops / 1e9:.1f} GFLOP in {secs:.1f} s)",
            "one_thread": {"value": round(f1 / s1 / 1e12, 5), "unit": "TFLOP/s",
                           "sample": f"the first {d1} shapes at batch 2 ({f1 / 1e9:.1f} GFLOP in {s1:.1f} s)"},
            "bandwidth_bound_steps": dict(hb, sample="weights of the 53 pruned-width layers with "
                                          f"{int(sparsity * 100)}% of every edge zeroed; activation gather on the inputs "
                                          "of layers 2-12 at batch 2 (bf16 bit patterns); bytes counted as for the GPU "
                                          "path (fp32 weights, bf16 activations) although the oracle holds fp64")}


# --------------------------------------------------------------------------------------------- #
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--reps", type=int, default=30, help="timed repetitions behind every median of the breakdown")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--sparsity", type=float, default=0.3, help="fraction of each edge zeroed in the sweep")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the weight gradients on the same stream as the input-gradient chain")
    ap.add_argument("--no-branch-overlap", action="store_true",
                    help="input gradients of the shortcut convolutions in line instead of on a side stream")
    ap.add_argument("--no-fused-lasso", action="store_true",
                    help="add the regulariser's gradient in a pass of its own after the weight gradients")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="only the timed step and its phases (no per-family timings)")
    ap.add_argument("--wgrad-streams", type=int, default=None, help="side streams the weight gradients alternate between")
    ap.add_argument("--layer-pass", metavar="FILE", default=None,
                    help="no timed step: launch every layer's calls one by one with a marker kernel between them "
                         "and write the list of calls to FILE (for a profiler run)")
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
    from paper_1901_09290_amd import profile_report as pr
    from paper_1901_09290_amd import workloads as wl

    B.lib()  # fail loudly if the HIP library is not built
    if args.wgrad_streams is not None:
        hz.WGRAD_STREAMS = args.wgrad_streams
    torch.cuda.set_device(0)
    N = args.batch

    def copy_probe():
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.neg(src, out=dst)       # one launch: 2^30 bytes read, 2^30 bytes written
        torch.cuda.synchronize()
        return {"kernel": "torch.neg (vectorized elementwise)", "read_bytes": 1 << 30, "write_bytes": 1 << 30}

    # ---- synthetic workloads ------------------------------------------------------------------ #
    full_specs, edges = wl.resnet50_layers(N=N)
    keep = wl.pruned_keep_sets(edges, seed=3)
    pruned_specs, pruned_edges = wl.with_widths(full_specs, edges, [k.size for k in keep])

    if args.layer_pass:
        layer_pass(args, torch, B, hz, wl, pr, full_specs, edges, pruned_specs, keep, copy_probe)
        return

    full = hz.Network(hz.build_network(full_specs, seed=2))
    pruned = hz.Network(hz.build_network(pruned_specs, seed=3))
    full.overlap_wgrad = pruned.overlap_wgrad = not args.no_overlap
    full.fuse_lasso = pruned.fuse_lasso = not args.no_fused_lasso
    full.overlap_branches = pruned.overlap_branches = not args.no_branch_overlap
    full.batch_branches_fwd = pruned.batch_branches_fwd = not args.no_branch_overlap and os.environ.get('PT_NOPAIR') is None
    rng = np.random.Generator(np.random.PCG64(10 + int(round(args.sparsity * 10))))
    zero_sets = wl.zeroed_channel_sets(pruned_edges, args.sparsity, rng)
    rweights = wl.network_weights(pruned_specs, pruned_edges, zero_sets, rng)
    rmodel = hz.ReconfigModel(pruned_specs, pruned_edges, rweights, seed=11)
    torch.cuda.synchronize()
    f_full, f_pruned = full.step_flops, pruned.step_flops
    log(f"full: {f_full / 1e12:.3f} TFLOP/step, pruned: {f_pruned / 1e12:.3f} TFLOP/step, "
        f"mem {torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    # ---- eager warm-up (also the first launches that set kernel attributes) ---------------------- #
    for _ in range(3):
        full.train_step(LAMBDA)
        rmodel.sweep(THRESHOLD)
        pruned.train_step(LAMBDA)
    torch.cuda.synchronize()
    counts0 = rmodel.new_counts.copy()
    expect = np.array([e.n - z.size for e, z in zip(pruned_edges, zero_sets)])
    assert np.array_equal(counts0, expect), "survivor counts differ from the zero pattern that was planted"

    use_graph = not args.no_graph
    side = torch.cuda.Stream()

    def graphed(fn):
        """fn as a replayable HIP graph (or fn itself with --no-graph)."""
        if not use_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                fn()
        torch.cuda.synchronize()
        return g.replay

    if use_graph:
        g1 = graphed(lambda: (full.train_step(LAMBDA), rmodel.detect(THRESHOLD)))
        g2 = graphed(lambda: (rmodel.compact(counts0), pruned.train_step(LAMBDA)))

        counts_host = torch.empty(rmodel.counts.numel(), dtype=rmodel.counts.dtype, pin_memory=True)

        def step():
            g1()
            counts_host.copy_(rmodel.counts, non_blocking=True)   # the sweep's one synchronising read-back
            torch.cuda.current_stream().synchronize()
            if not np.array_equal(counts_host.numpy(), counts0):
                raise RuntimeError("survivor counts changed between steps")
            g2()
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
    marks = [ev() for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_step = marks[0].elapsed_time(marks[-1]) / args.steps
    ms_step_median = float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]))
    value = (f_full + f_pruned) / (ms_step * 1e-3) / 1e12

    # ---- medians of the phases and the kernel families ------------------------------------------ #
    flush_buf = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")    # 1 GiB: four times the last-level cache

    def flush():
        flush_buf.zero_()

    def median_ms(fn, reps=None, inner=1, cold=False):
        """Median over reps of the time of `inner` back-to-back calls of fn, per call.  cold: a 1 GiB fill runs
        before every repetition (outside its events) so nothing fn reads is still in a cache."""
        reps = args.reps if reps is None else reps
        fn()
        pairs = []
        for _ in range(reps):
            if cold:
                flush()
            a, b = ev(), ev()
            a.record()
            for _ in range(inner):
                fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in pairs])) / inner

    r_full, r_pruned = graphed(lambda: full.train_step(LAMBDA)), graphed(lambda: pruned.train_step(LAMBDA))
    r_detect, r_compact = graphed(lambda: rmodel.detect(THRESHOLD)), graphed(lambda: rmodel.compact(counts0))
    t_full, t_pruned = median_ms(r_full), median_ms(r_pruned)
    t_detect, t_compact = median_ms(r_detect, inner=4), median_ms(r_compact, inner=2)

    if args.quick:
        print(json.dumps({"value": round(value, 3), "ms_per_step": round(ms_step, 4), "full_ms": round(t_full, 4),
                          "pruned_ms": round(t_pruned, 4), "detect_ms": round(t_detect, 4),
                          "compact_ms": round(t_compact, 4), "wgrad_streams": hz.WGRAD_STREAMS}), flush=True)
        return
    t_detect_cold, t_compact_cold = median_ms(r_detect, cold=True), median_ms(r_compact, cold=True)

    # kernel families: every layer's call of one kind back to back, as one graph on the timing stream
    nets = {"full": full, "pruned": pruned}
    fam = {}
    for tag, net in nets.items():
        L = net.layers
        f = fam[tag] = {}
        f["fwd"] = median_ms(graphed(lambda: [l.fwd(net.ws) for l in L]))
        f["bwd_data"] = median_ms(graphed(lambda: [l.bwd_data_crsk() for l in L]))
        f["bwd_weight"] = median_ms(graphed(lambda: [l.bwd_weight(net.ws) for l in L]))
        f["bwd_weight_lasso"] = median_ms(graphed(lambda: [l.bwd_weight_lasso(net.ws, LAMBDA) for l in L]))
        r = graphed(lambda: B.group_norms_batched(net.norm_jobs, net.ws_norms))
        f["group_norms"], f["group_norms_cold"] = median_ms(r, inner=4), median_ms(r, cold=True)
        r = graphed(lambda: B.group_lasso_grad_batched(net.lasso_jobs, LAMBDA))
        f["group_lasso_grad"], f["group_lasso_grad_cold"] = median_ms(r, inner=4), median_ms(r, cold=True)
        # not part of the timed step: the optimizer step with the regulariser folded in (lr = 0: weights unchanged)
        f["optimizer_step_fused"] = median_ms(graphed(lambda: net.optimizer_step(LAMBDA, 0.0, 0.9, 1e-4)), inner=2)
        # not part of the timed step either: feature normalisation of every convolution output, forward and backward
        f["fwd+bn"] = median_ms(lambda: net.fwd_bn_all(False), reps=5)
        f["fwd+bn_fused"] = median_ms(lambda: net.fwd_bn_all(True), reps=5)
        f["bn_fwd"] = median_ms(net.bn_fwd_all, reps=5)
        f["bn_bwd"] = median_ms(net.bn_bwd_all, reps=5)

    def fam_sum(tag, kind, fn):
        return sum(fn(l.spec, kind) for l in nets[tag].layers if has_call(l.spec, kind))
    fl = {t: {k: fam_sum(t, k, lambda s, _k: s.flops) for k in CONV_KINDS} for t in nets}
    by = {t: {k: fam_sum(t, k, conv_bytes) for k in CONV_KINDS} for t in nets}
    roof = {t: {k: fam_sum(t, k, conv_roof_s) for k in CONV_KINDS} for t in nets}
    params = {t: sum(l.spec.params for l in nets[t].layers) for t in nets}

    # dominant kernel of the step: k_igemm_dl serves conv_fwd and conv_bwd_data, k_wgrad_dl (+ its reduction pass)
    # conv_bwd_weight; the one with the larger time over both widths is reported against its roof
    tot = {k: fam["full"][k] + fam["pruned"][k] for k in CONV_KINDS}
    kernels = {"k_igemm_dl (conv_fwd + conv_bwd_data launches; the first layer's forward is k_stem_fwd, early 3x3 layers take k_conv3x3_res)": ("fwd", "bwd_data"),
               "k_wgrad_dl + k_wgrad_reduce (conv_bwd_weight launches)": ("bwd_weight",)}
    dom_kernel = max(kernels, key=lambda k: sum(tot[f] for f in kernels[k]))
    fams = kernels[dom_kernel]

    # one launch per call: the stride-parity classes of a strided input gradient share a launch
    n_launch = sum(1 for f in fams for net in nets.values() for l in net.layers if has_call(l.spec, f))
    dom_flops = sum(fl[t][f] for f in fams for t in nets)
    dom_bytes = sum(by[t][f] for f in fams for t in nets)
    dom_s = sum(tot[f] for f in fams) * 1e-3
    # which roof bounds this kernel on this workload: time at the HBM peak vs time at the bf16 MFMA peak
    t_hbm, t_mfma = dom_bytes / (PEAK_HBM_GBS * 1e9), dom_flops / (PEAK_BF16_TFLOPS * 1e12)
    t_roof = sum(roof[t][f] for f in fams for t in nets)
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

    # HBM traffic of the dominant kernel comes from hardware counters, which need runs of their own under the
    # profiler: the summary written from those runs names the kernel sources it was taken with, and the figure is
    # reported only while those sources are the ones this run uses
    tr = pr.read_traffic(os.path.join(ROOT, "profiles", pr.TRAFFIC_FILE), "igemm" if "k_igemm_dl" in dom_kernel else "wgrad")
    if tr is not None and tr["digest"] == pr.source_digest():
        roofline["traffic"] = tr["bytes_per_launch"]
        roofline["traffic_unit"] = "bytes per launch (scaled FETCH_SIZE + WRITE_SIZE, profiles/" + pr.TRAFFIC_FILE + ")"
    else:
        roofline["traffic_note"] = ("no counter summary for these kernel sources" if tr is None or tr["digest"] is None
                                    else "the counter summary in profiles/ was taken with other kernel sources")

    ab = rmodel.algorithmic_bytes()
    sweep_bytes = sum(ab.values())
    t_sweep = t_detect + t_compact

    # activation gather, counted two ways: strictly (survivors read once and written once) and at the granularity
    # the memory system moves (every 64-byte segment of a source row holds a survivor, so whole rows are read)
    act_strict = ab["compact_nhwc"]
    act_rows = sum(2 * s.N * s.H * s.W * (s.C + int(counts0[s.in_edge])) for s in pruned_specs if s.in_edge is not None)
    keep_frac = act_strict / 2 / (act_rows - act_strict / 2)          # f = survivors / source channels, byte-weighted
    r_act = graphed(lambda: rmodel.compact_activations(counts0))
    t_act, t_act_cold = median_ms(r_act, inner=2), median_ms(r_act, cold=True)

    def hbm(nbytes, ms):
        return {"ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}

    def fam_table(tag):
        out = {}
        for k in CONV_KINDS:
            t = fam[tag][k]
            out[k] = {"ms": round(t, 4), "tflops": round(fl[tag][k] / (t * 1e-3) / 1e12, 1),
                      "algorithmic_GBps": round(by[tag][k] / (t * 1e-3) / 1e9, 1),
                      "per_layer_roof_ms": round(roof[tag][k] * 1e3, 4),
                      "frac_of_per_layer_roof": round(roof[tag][k] * 1e3 / t, 4)}
        # what the step launches when the regulariser's gradient is folded into the weight gradient (the default)
        t = fam[tag]["bwd_weight_lasso"]
        out["bwd_weight_with_lasso"] = {"ms": round(t, 4), "tflops": round(fl[tag]["bwd_weight"] / (t * 1e-3) / 1e12, 1),
                                        "frac_of_per_layer_roof": round(roof[tag]["bwd_weight"] * 1e3 / t, 4)}
        t3 = sum(fam[tag][k] for k in CONV_KINDS)
        out["all_three"] = {"ms": round(t3, 4), "frac_of_per_layer_roof": round(sum(roof[tag].values()) * 1e3 / t3, 4)}
        out["group_norms"] = dict(hbm(6 * params[tag], fam[tag]["group_norms"]),
                                  cold=hbm(6 * params[tag], fam[tag]["group_norms_cold"]))
        out["group_lasso_grad(separate pass)"] = dict(hbm(12 * params[tag], fam[tag]["group_lasso_grad"]),
                                                      cold=hbm(12 * params[tag], fam[tag]["group_lasso_grad_cold"]))
        out["optimizer_step_fused(not in step)"] = hbm(20 * params[tag], fam[tag]["optimizer_step_fused"])
        out["fwd+bn(not in step)"] = {"separate_ms": round(fam[tag]["fwd+bn"], 4),
                                      "statistics_in_conv_epilogue_ms": round(fam[tag]["fwd+bn_fused"], 4)}
        for k, bpe in (("bn_fwd", 6), ("bn_bwd", 10)):
            out[k + "(not in step)"] = hbm(bpe * nets[tag].bn_elements, fam[tag][k])
        return out

    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-50 conv layers (53), batch {N}, 224x224, NHWC bf16: train step at full width "
                               f"(cfg3) + reconfiguration sweep at {int(args.sparsity * 100)}% zeroed groups (cfg5) + "
                               "train step at ragged pruned widths (cfg4)",
                   "lambda": LAMBDA, "threshold": THRESHOLD, "hip_graphs": use_graph,
                   "wgrad_side_streams": 0 if args.no_overlap else hz.WGRAD_STREAMS,
                   "shortcut_input_gradients_on_side_streams": bool(full.overlap_branches and full.overlap_wgrad),
                   "lasso_in_wgrad_reduce": bool(full.fuse_lasso and full.overlap_wgrad),
                   "kernel_sources": pr.source_digest()},
        "roofline": roofline,
        "breakdown": {
            "timing": f"medians of {args.reps} repetitions (HIP events around graph replays); 'cold' = a 1 GiB fill "
                      "before every repetition, and the event-to-event time of a single replay",
            "ms_per_step_median": round(ms_step_median, 4),
            "wall_ms_per_step": round(wall_ms, 4),
            "full_width": {"ms": round(t_full, 4), "tflops": round(f_full / (t_full * 1e-3) / 1e12, 2),
                           "frac_mfma_peak": round(f_full / (t_full * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                           "frac_of_per_layer_roof": round(sum(roof["full"].values()) * 1e3 / t_full, 4)},
            "pruned_width": {"ms": round(t_pruned, 4), "tflops": round(f_pruned / (t_pruned * 1e-3) / 1e12, 2),
                             "frac_mfma_peak": round(f_pruned / (t_pruned * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                             "frac_of_per_layer_roof": round(sum(roof["pruned"].values()) * 1e3 / t_pruned, 4),
                             "flop_ratio_vs_full": round(f_pruned / f_full, 4),
                             "time_ratio_vs_full": round(t_pruned / t_full, 4)},
            "kernel_families_full": fam_table("full"),
            "kernel_families_pruned": fam_table("pruned"),
            "reconfig_sweep": dict(hbm(sweep_bytes, t_sweep), detect_ms=round(t_detect, 4), compact_ms=round(t_compact, 4),
                                   cold=dict(hbm(sweep_bytes, t_detect_cold + t_compact_cold),
                                             detect_ms=round(t_detect_cold, 4), compact_ms=round(t_compact_cold, 4)),
                                   algorithmic_MB={k: round(v / 1e6, 1) for k, v in ab.items()},
                                   activation_gather={
                                       "strict": dict(hbm(act_strict, t_act), cold=hbm(act_strict, t_act_cold)),
                                       "whole_source_rows": dict(hbm(act_rows, t_act), cold=hbm(act_rows, t_act_cold)),
                                       "keep_fraction": round(keep_frac, 4),
                                       "strict_ceiling_2f_over_1_plus_f": round(2 * keep_frac / (1 + keep_frac), 4)}),
        },
    }
    if args.copy_probe:
        out["copy_probe"] = copy_probe()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.sparsity)
    print(json.dumps(out), flush=True)


# --------------------------------------------------------------------------------------------- #
def layer_pass(args, torch, B, hz, wl, pr, full_specs, edges, pruned_specs, keep, copy_probe):
    """Every convolution call of three networks (full widths, the ragged pruned widths, and the pruned widths
    rounded up to the next multiple of 64 channels), one layer at a time on one stream, in network order, eagerly.
    A marker kernel (pt_zero_groups on 64 elements) follows every call and three in a row open the pass, so that a
    kernel trace of this run splits into calls without knowing how many kernels a call launches."""
    up64 = [(k.size + 63) // 64 * 64 for k in keep]
    padded_specs, _ = wl.with_widths(full_specs, edges, up64)
    nets = [("full", full_specs, 2), ("pruned", pruned_specs, 3), ("pruned_up64", padded_specs, 4)]
    mark_in = torch.ones(64, dtype=torch.float32, device="cuda:0")
    mark_out = torch.zeros(64, dtype=torch.uint8, device="cuda:0")

    def marker():
        B.zero_groups(mark_in, 64, 0.5, mark_out)

    calls = []
    for tag, specs, seed in nets:
        net = hz.Network(hz.build_network(specs, seed=seed))
        B.group_norms_batched(net.norm_jobs, net.ws_norms)
        B.weights_to_crsk_batched(net.crsk_jobs)
        todo = [("fwd", lambda l: l.fwd(net.ws)), ("bwd_data", lambda l: l.bwd_data_crsk()),
                ("bwd_weight", lambda l: l.bwd_weight(net.ws)),
                ("bwd_weight_lasso", lambda l: l.bwd_weight_lasso(net.ws, LAMBDA))]
        for _kind, fn in todo:                     # untimed first launches (kernel attributes, code upload)
            for l in net.layers:
                fn(l)
        torch.cuda.synchronize()
        for _ in range(3):
            marker()
        for kind, fn in todo:
            for l in net.layers:
                if not has_call(l.spec, kind):
                    continue
                fn(l)
                marker()
                s = l.spec
                calls.append({"net": tag, "kind": kind, "layer": s.name, "shape": list(s.shape_key()),
                              "flops": s.flops, "bytes": conv_bytes(s, kind)})
        torch.cuda.synchronize()
        del net
        torch.cuda.empty_cache()
    man = {"batch": args.batch, "marker": "k_zero_groups", "nets": [t for t, _, _ in nets], "calls": calls,
           "kernel_sources": pr.source_digest(), "peak_bf16_tflops": PEAK_BF16_TFLOPS, "peak_hbm_GBps": PEAK_HBM_GBS}
    if args.copy_probe:
        man["copy_probe"] = copy_probe()
    os.makedirs(os.path.dirname(os.path.abspath(args.layer_pass)), exist_ok=True)
    with open(args.layer_pass, "w") as f:
        json.dump(man, f)
    print(json.dumps({"layer_pass": args.layer_pass, "calls": len(calls)}), flush=True)


if __name__ == "__main__":
    main()
