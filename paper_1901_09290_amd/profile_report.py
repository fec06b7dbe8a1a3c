"""Text summaries of rocprofv3 runs of bench.py: per-layer roofline table, MFMA counters, HBM traffic, step trace.

Host-side text processing only (csv in, text out); nothing here touches the GPU or the library.

    python -m paper_1901_09290_amd.profile_report layers  --manifest M.json --trace T_kernel_trace.csv
                                                          [--fetch F_counter_collection.csv --write W_counter_collection.csv] --out FILE
    python -m paper_1901_09290_amd.profile_report traffic --manifest M.json --fetch F.csv --write W.csv --out FILE
    python -m paper_1901_09290_amd.profile_report mfma    --manifest M.json --trace T.csv --pmc P_counter_collection.csv --out FILE
    python -m paper_1901_09290_amd.profile_report step    --stats S_kernel_stats.csv --bench BENCH.json --out FILE

M.json is what `bench.py --layer-pass M.json` writes: the list of convolution calls it launched, one marker kernel
after each call and three markers in front of every network's pass.  The csv files come from rocprofv3 runs of that
same command (kernel trace, or one counter collection per run).
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import re
import sys
from typing import Dict, List, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = "bench_resnet50_b64_hbm_traffic.txt"
MFMA_FLOP_PER_MOP = 512        # SQ_INSTS_VALU_MFMA_MOPS_* count units of 512 floating-point operations


def source_digest() -> str:
    """Fingerprint of the kernel sources (every file under csrc/), to tie a counter summary to the code it measured."""
    h = hashlib.sha256()
    d = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def read_traffic(path: str, which: str) -> Optional[Dict[str, object]]:
    """The per-launch HBM traffic line of the traffic summary ('igemm' or 'wgrad') and the source digest it names."""
    if not os.path.exists(path):
        return None
    text = open(path).read()
    pat = (r"per k_igemm_dl launch .*?= ([0-9.]+) MB of HBM traffic" if which == "igemm"
           else r"per pt_conv_bwd_weight call .*?= ([0-9.]+) MB of HBM traffic")
    m = re.search(pat, text)
    if not m:
        return None
    d = re.search(r"kernel sources: ([0-9a-f]{16})", text)
    return {"bytes_per_launch": float(m.group(1)) * 1e6, "digest": d.group(1) if d else None}


# --------------------------------------------------------------------------------------------- #
def short(name: str) -> str:
    n = re.sub(r"^void ", "", name)
    n = re.sub(r"\(.*", "", n)
    return n.replace("pt::", "")


MAIN_FAMILIES = ("k_igemm_dl", "k_wgrad_dl", "k_igemm", "k_wgrad", "k_stem_fwd", "k_stem_wgrad", "k_conv3x3_res")


def family(n: str) -> Optional[str]:
    for f in ("k_igemm_dl", "k_igemm", "k_conv3x3_res", "k_stem_fwd", "k_stem_wgrad_reduce", "k_stem_wgrad", "k_wgrad_dl", "k_wgrad_reduce", "k_wgrad",
              "k_zero_class"):
        if n.startswith(f + "<") or n == f or n.startswith(f + "4"):
            return "k_wgrad_reduce" if f in ("k_wgrad_reduce", "k_stem_wgrad_reduce") else f
    return None


def load_trace(path: str) -> List[dict]:
    rows = []
    for r in csv.DictReader(open(path)):
        rows.append({"id": int(r["Dispatch_Id"]), "name": short(r["Kernel_Name"]),
                     "t0": int(r["Start_Timestamp"]), "t1": int(r["End_Timestamp"])})
    rows.sort(key=lambda r: r["id"])
    return rows


def load_counters(path: str) -> List[dict]:
    """One record per dispatch with a dict of its counters (a run collects one or several counters)."""
    by: Dict[int, dict] = {}
    for r in csv.DictReader(open(path)):
        d = by.setdefault(int(r["Dispatch_Id"]), {"id": int(r["Dispatch_Id"]), "name": short(r["Kernel_Name"]), "c": {}})
        d["c"][r["Counter_Name"]] = d["c"].get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return [by[k] for k in sorted(by)]


def split_calls(rows: List[dict], manifest: dict) -> List[List[dict]]:
    """The dispatches of every call of the manifest: each network's pass opens with three markers in a row, and one
    marker closes every call."""
    mk = manifest["marker"]
    per_net = collections.OrderedDict()
    for c in manifest["calls"]:
        per_net[c["net"]] = per_net.get(c["net"], 0) + 1
    starts = [i + 3 for i in range(len(rows) - 2) if all(rows[i + j]["name"] == mk for j in range(3))
              and (i == 0 or rows[i - 1]["name"] != mk)]
    if len(starts) != len(per_net):
        raise SystemExit(f"expected {len(per_net)} marker triples in the trace, found {len(starts)}")
    out = []
    for start, (net, n_calls) in zip(starts, per_net.items()):
        i, cur = start, []
        got = 0
        while got < n_calls:
            if i >= len(rows):
                raise SystemExit(f"trace ends inside the pass of network {net}")
            if rows[i]["name"] == mk:
                out.append(cur)
                cur = []
                got += 1
            else:
                cur.append(rows[i])
            i += 1
    assert len(out) == len(manifest["calls"])
    return out


def probe_factor(rows: List[dict], counter: str, manifest: dict) -> float:
    """Bytes per counter unit: the copy probe moves a known number of bytes through a plain elementwise kernel."""
    p = manifest.get("copy_probe")
    if not p:
        raise SystemExit("the manifest has no copy probe (run bench.py --layer-pass with --copy-probe)")
    vals = [r["c"][counter] for r in rows if "elementwise" in r["name"] and "neg" in r["name"] and counter in r["c"]]
    if not vals:
        raise SystemExit("the copy probe's kernel is not in the counter file")
    want = p["read_bytes"] if counter == "FETCH_SIZE" else p["write_bytes"]
    return want / (sum(vals) / len(vals))


# --------------------------------------------------------------------------------------------- #
def cmd_layers(a) -> None:
    man = json.load(open(a.manifest))
    calls = man["calls"]
    segs = split_calls(load_trace(a.trace), man)
    hbm, mfma = man["peak_hbm_GBps"] * 1e9, man["peak_bf16_tflops"] * 1e12
    traffic = None
    if a.fetch and a.write:
        fr, wr = load_counters(a.fetch), load_counters(a.write)
        ff, wf = probe_factor(fr, "FETCH_SIZE", man), probe_factor(wr, "WRITE_SIZE", man)
        fs, ws = split_calls(fr, man), split_calls(wr, man)
        traffic = [sum(r["c"].get("FETCH_SIZE", 0) for r in f) * ff + sum(r["c"].get("WRITE_SIZE", 0) for r in w) * wf
                   for f, w in zip(fs, ws)]
    o = []
    o.append("Per-layer roofline table: every convolution call of the ResNet-50 conv stack at batch %d, NHWC bf16, on one MI355X" % man["batch"])
    o.append("kernel sources: %s" % man["kernel_sources"])
    o.append("commands (from /tmp, TMPDIR=/tmp; the csv files land under <out>):")
    o.append("  rocprofv3 --kernel-trace --output-format csv -d <out> -o lp -- python3 bench.py --layer-pass <out>/manifest.json --copy-probe")
    if traffic:
        o.append("  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out>/f -o f -- python3 bench.py --layer-pass <out>/f/manifest.json --copy-probe")
        o.append("  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out>/w -o w -- python3 bench.py --layer-pass <out>/w/manifest.json --copy-probe")
    o.append("  python3 -m paper_1901_09290_amd.profile_report layers --manifest ... --trace ..._kernel_trace.csv [--fetch ... --write ...] --out <this file>")
    o.append("One call = all kernels the entry point launches (conv_bwd_data: one launch per stride-parity class; conv_bwd_weight_lasso:")
    o.append("main kernel + reduction pass when the pixel axis is split).  us = sum of the kernels' durations in the trace (launch gaps")
    o.append("excluded); calls run one at a time in network order, so inputs are not cache-resident from a previous repetition.")
    o.append("GF = 2*N*P*Q*K*C*R*S per call; algorithmic bytes = x + y + w in bf16 once (bwd_weight: x + dy once, dw fp32 once; MB_fwd is")
    o.append("the forward call's); TF/s and GB/s are GF and algorithmic bytes over us.")
    o.append("roof = max(bytes / %.0f GB/s, GF / %.0f TFLOP/s); bound = which of the two; frac = roof / us." % (hbm / 1e9, mfma / 1e12))
    if traffic:
        o.append("traf = bytes the call's kernels move between the L2s and the fabric (FETCH_SIZE and WRITE_SIZE scaled by the copy probe; reads")
        o.append("that the Infinity Cache serves are counted too, e.g. weights that each of the eight L2s fetches for itself) / algorithmic bytes.")
    o.append("Networks: full = published widths; pruned = ragged widths (keep fraction U[0.4,0.9] per channel edge, never a multiple of 16);")
    o.append("pruned_up64 = the pruned widths rounded up to the next multiple of 64 (the padded twin of every pruned layer).")
    o.append("")
    rec = []
    for c, seg in zip(calls, segs):
        us = sum(r["t1"] - r["t0"] for r in seg) / 1e3
        t_h, t_m = c["bytes"] / hbm * 1e6, c["flops"] / mfma * 1e6
        rec.append(dict(c, us=us, n_k=len(seg), roof=max(t_h, t_m), bound="hbm" if t_h >= t_m else "mfma"))
    for i, r in enumerate(rec):
        r["traf"] = traffic[i] / r["bytes"] if traffic else None
    idx = {(r["net"], r["kind"], r["layer"]): r for r in rec}
    kinds = ("fwd", "bwd_data", "bwd_weight_lasso")
    short_kind = {"fwd": "fwd", "bwd_data": "bwd_data", "bwd_weight_lasso": "bwd_weight (regulariser folded in)"}
    for net in ("full", "pruned"):
        layers = [r["layer"] for r in rec if r["net"] == net and r["kind"] == "fwd"]
        if not layers:
            continue
        twin = net == "pruned"
        o.append("== %s widths: one row per layer, then per call: %s ==" % (net, "us TF/s GB/s frac bound(h=hbm,m=mfma)" + (" traf" if traffic else "")
                                                                       + (" t/t64 (time / time of the padded twin)" if twin else "")))
        o.append("%-15s %-26s %7s %7s | %s" % ("layer", "H,W,C,K,R,stride", "GF", "MB_fwd", " | ".join("%-*s" % (31 + (5 if traffic else 0) + (5 if twin else 0), short_kind[k][:36]) for k in kinds)))
        for name in layers:
            f = idx[(net, "fwd", name)]
            sh = f["shape"]
            cells = []
            for k in kinds:
                r = idx.get((net, k, name))
                width = 31 + (5 if traffic else 0) + (5 if twin else 0)
                if r is None:
                    cells.append("%-*s" % (width, "-"))
                    continue
                c = "%6.1f %4.0f %5.0f %5.3f %s" % (r["us"], r["flops"] / r["us"] / 1e6, r["bytes"] / r["us"] / 1e3, r["roof"] / r["us"], r["bound"][0])
                if traffic:
                    c += " %4.2f" % r["traf"]
                if twin:
                    tw = idx.get(("pruned_up64", k, name))
                    c += " %4.2f" % (r["us"] / tw["us"]) if tw else "    -"
                cells.append("%-*s" % (width, c))
            o.append("%-15s %-26s %7.2f %7.2f | %s" % (name, "%d,%d,%d,%d,%d,%d" % (sh[1], sh[2], sh[3], sh[4], sh[5], sh[7]), f["flops"] / 1e9,
                                                    f["bytes"] / 1e6, " | ".join(cells)))
        for k in kinds:
            rows = [r for r in rec if r["net"] == net and r["kind"] == k]
            us, roof = sum(r["us"] for r in rows), sum(r["roof"] for r in rows)
            fl, by = sum(r["flops"] for r in rows), sum(r["bytes"] for r in rows)
            o.append("total %-34s %4d calls %8.1f GF %8.1f MB %8.1f us %5.0f TF/s %5.0f GB/s; sum of the layers' roofs %7.1f us -> fraction %.3f%s" % (
                short_kind[k], len(rows), fl / 1e9, by / 1e6, us, fl / us / 1e6, by / us / 1e3, roof, roof / us,
                ("; measured / algorithmic traffic %.2f" % (sum(traffic[i] for i, r in enumerate(rec) if r["net"] == net and r["kind"] == k) / by)) if traffic else ""))
        rows = [r for r in rec if r["net"] == net and r["kind"] == "bwd_weight"]
        if rows:
            o.append("      (the weight gradient without the regulariser, same layers: %.1f us)" % sum(r["us"] for r in rows))
        o.append("")
    # ragged widths against their padded twins
    o.append("== ragged widths against their padded twins (pruned vs pruned_up64, same layer, same call) ==")
    o.append("A ragged layer has fewer FLOPs and fewer bytes than its twin; it should never take longer.  time ratio = pruned us / twin us,")
    o.append("next to the FLOP and algorithmic-byte ratios of the two networks; then the layers that take more than 1.15x their twin's time.")
    for kind in kinds:
        pr_ = [r for r in rec if r["net"] == "pruned" and r["kind"] == kind]
        tw_ = [idx[("pruned_up64", kind, r["layer"])] for r in pr_]
        if not pr_:
            continue
        tp, tt = sum(r["us"] for r in pr_), sum(r["us"] for r in tw_)
        fp, ft = sum(r["flops"] for r in pr_), sum(r["flops"] for r in tw_)
        bp, bt = sum(r["bytes"] for r in pr_), sum(r["bytes"] for r in tw_)
        slower = sorted(((r["us"] / t["us"], r["layer"]) for r, t in zip(pr_, tw_) if r["us"] > 1.15 * t["us"]), reverse=True)
        o.append("%-17s time ratio %.3f (FLOP ratio %.3f, byte ratio %.3f); slower than 1.15x the twin: %d of %d layers%s" % (
            kind, tp / tt, fp / ft, bp / bt, len(slower), len(pr_),
            (" (" + ", ".join("%s x%.2f" % (n, x) for x, n in slower[:6]) + ")") if slower else ""))
    _write(a.out, o)


def cmd_traffic(a) -> None:
    man = json.load(open(a.manifest))
    fr, wr = load_counters(a.fetch), load_counters(a.write)
    ff, wf = probe_factor(fr, "FETCH_SIZE", man), probe_factor(wr, "WRITE_SIZE", man)
    fs, ws = split_calls(fr, man), split_calls(wr, man)
    o = []
    o.append("rocprofv3 --pmc HBM traffic summary: the convolution kernels on the ResNet-50 conv layers at batch %d (eager launches, one call at a time)" % man["batch"])
    o.append("kernel sources: %s" % man["kernel_sources"])
    o.append("commands (from /tmp, TMPDIR=/tmp), one counter per run:")
    o.append("  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out>/f -o f -- python3 bench.py --layer-pass <out>/f/manifest.json --copy-probe")
    o.append("  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out>/w -o w -- python3 bench.py --layer-pass <out>/w/manifest.json --copy-probe")
    o.append("  python3 -m paper_1901_09290_amd.profile_report traffic --manifest <out>/f/manifest.json --fetch <out>/f/..._counter_collection.csv --write <out>/w/..._counter_collection.csv --out <this file>")
    o.append("Scale factors from the copy probe (a plain elementwise kernel that reads 1 GiB and writes 1 GiB):")
    o.append("  FETCH_SIZE: %.1f bytes per unit;  WRITE_SIZE: %.1f bytes per unit" % (ff, wf))
    o.append("The counters see what the L2s exchange with the fabric: reads served by the Infinity Cache (256 MB) are counted like HBM reads.")
    o.append("Only the calls of the two networks the benchmark's step runs (full and pruned widths) are counted below.")
    o.append("")
    agg = collections.defaultdict(lambda: [0, 0.0, 0.0])
    per_kind = collections.defaultdict(lambda: [0, 0, 0.0, 0.0, 0.0])   # calls, launches, fetch, write, algorithmic
    for c, f, w in zip(man["calls"], fs, ws):
        if c["net"] not in ("full", "pruned"):
            continue
        for r in f:
            agg[r["name"]][0] += 1
            agg[r["name"]][1] += r["c"].get("FETCH_SIZE", 0) * ff
        for r in w:
            agg[r["name"]][2] += r["c"].get("WRITE_SIZE", 0) * wf
        k = per_kind["igemm" if c["kind"] in ("fwd", "bwd_data") else "wgrad"]
        k[0] += 1
        k[1] += len(f)
        k[2] += sum(r["c"].get("FETCH_SIZE", 0) for r in f) * ff
        k[3] += sum(r["c"].get("WRITE_SIZE", 0) for r in w) * wf
        k[4] += c["bytes"]
    o.append("%-66s %8s %15s %15s" % ("kernel", "launches", "fetch_MB/launch", "write_MB/launch"))
    for n in sorted(agg, key=lambda n: -(agg[n][1] + agg[n][2])):
        c = agg[n]
        o.append("%-66s %8d %15.2f %15.2f" % (n[:66], c[0], c[1] / c[0] / 1e6, c[2] / c[0] / 1e6))
    o.append("")
    k = per_kind["wgrad"]
    if k[0]:
        o.append("per pt_conv_bwd_weight call (main kernel + reduction pass where the pixel axis is split, %d calls): fetch %.1f MB + write %.1f MB = %.1f MB of HBM traffic"
                 % (k[0], k[2] / k[0] / 1e6, k[3] / k[0] / 1e6, (k[2] + k[3]) / k[0] / 1e6))
        o.append("algorithmic bytes per call (x + dy read once, dw written once): %.1f MB  -> traffic / algorithmic = %.2f"
                 % (k[4] / k[0] / 1e6, (k[2] + k[3]) / k[4]))
    k = per_kind["igemm"]
    if k[0]:
        o.append("per k_igemm_dl launch (conv_fwd and conv_bwd_data calls, %d launches, the first layer's k_stem_fwd, the early 3x3 layers' k_conv3x3_res and the zero fill of empty parity classes included): fetch %.1f MB + write %.1f MB = %.1f MB of HBM traffic"
                 % (k[1], k[2] / k[1] / 1e6, k[3] / k[1] / 1e6, (k[2] + k[3]) / k[1] / 1e6))
        o.append("algorithmic bytes per launch: %.1f MB  -> traffic / algorithmic = %.2f" % (k[4] / k[1] / 1e6, (k[2] + k[3]) / k[4]))
    _write(a.out, o)


def cmd_mfma(a) -> None:
    man = json.load(open(a.manifest))
    tr, pm = load_trace(a.trace), load_counters(a.pmc)
    tsegs, psegs = split_calls(tr, man), split_calls(pm, man)
    peak = man["peak_bf16_tflops"] * 1e12
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    for c, ts, ps in zip(man["calls"], tsegs, psegs):
        if c["net"] not in ("full", "pruned") or len(ts) != len(ps):
            continue
        main = [r for r in ts if family(r["name"]) in MAIN_FAMILIES]
        for t, p in zip(ts, ps):
            if family(t["name"]) not in MAIN_FAMILIES:
                continue
            g = agg[(c["net"], t["name"])]
            g["n"] += 1
            g["us"] += (t["t1"] - t["t0"]) / 1e3
            g["flops"] += c["flops"] / max(1, len(main))
            for k, v in p["c"].items():
                g[k] += v
            g["util_us"] += p["c"].get("MfmaUtil", 0.0) * (t["t1"] - t["t0"]) / 1e3
    o = []
    o.append("rocprofv3 --pmc MFMA summary: the convolution kernels on the ResNet-50 conv layers at batch %d, per kernel instantiation and width" % man["batch"])
    o.append("kernel sources: %s" % man["kernel_sources"])
    o.append("commands (from /tmp, TMPDIR=/tmp); durations come from the kernel-trace run, counters from the counter run of the same command:")
    o.append("  rocprofv3 --kernel-trace --output-format csv -d <out> -o lp -- python3 bench.py --layer-pass <out>/manifest.json --copy-probe")
    o.append("  rocprofv3 --pmc SQ_INSTS_VALU_MFMA_MOPS_BF16 MfmaUtil --output-format csv -d <out>/m -o m -- python3 bench.py --layer-pass <out>/m/manifest.json")
    o.append("  python3 -m paper_1901_09290_amd.profile_report mfma --manifest <out>/manifest.json --trace <out>/..._kernel_trace.csv --pmc <out>/m/..._counter_collection.csv --out <this file>")
    o.append("mfma_GF = SQ_INSTS_VALU_MFMA_MOPS_BF16 x %d / 1e9 per launch (what the matrix cores executed, tile padding included);" % MFMA_FLOP_PER_MOP)
    o.append("alg_GF = the layer's 2*N*P*Q*K*C*R*S per launch; pad = mfma_GF / alg_GF; TF/s = mfma_GF / us; %%peak = TF/s / %.0f;" % (peak / 1e12))
    o.append("busy% = MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES summed over the SIMDs / (GRBM_GUI_ACTIVE x number of SIMDs): the share of the kernel's")
    o.append("cycles in which a SIMD's matrix core was executing, averaged over the launches with their durations as weights.")
    o.append("")
    o.append("%-7s %-52s %6s %8s %9s %9s %5s %7s %6s %6s" % ("width", "kernel", "calls", "avg_us", "alg_GF", "mfma_GF", "pad", "TF/s", "%peak", "busy%"))
    keys = sorted(agg, key=lambda k: (k[0], -agg[k]["us"]))
    tot = collections.defaultdict(lambda: collections.defaultdict(float))
    for key in keys:
        g = agg[key]
        mf = g.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0) * MFMA_FLOP_PER_MOP
        busy = g["util_us"] / g["us"] / 100
        o.append("%-7s %-52s %6d %8.2f %9.2f %9.2f %5.2f %7.0f %6.1f %6.1f" % (
            key[0], key[1][:52], g["n"], g["us"] / g["n"], g["flops"] / g["n"] / 1e9, mf / g["n"] / 1e9,
            mf / max(1.0, g["flops"]), mf / g["us"] / 1e6, 100 * mf / (g["us"] * 1e-6) / peak, 100 * busy))
        t = tot[(key[0], family(key[1]))]
        for k, v in g.items():
            t[k] += v
    o.append("")
    for key in sorted(tot):
        g = tot[key]
        mf = g.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0) * MFMA_FLOP_PER_MOP
        busy = g["util_us"] / g["us"] / 100
        o.append("%-7s %-12s all instantiations: %5d launches, %8.1f us; executed %.1f TFLOP/s on the matrix cores = %.1f%% of the bf16 peak (algorithmic %.1f TFLOP/s); MFMA busy %.1f%%" % (
            key[0], key[1], g["n"], g["us"], mf / g["us"] / 1e6, 100 * mf / (g["us"] * 1e-6) / peak, g["flops"] / g["us"] / 1e6, 100 * busy))
    _write(a.out, o)


def cmd_step(a) -> None:
    rows = list(csv.DictReader(open(a.stats)))
    bench = json.loads(open(a.bench).read().strip().splitlines()[-1])
    o = []
    o.append("rocprofv3 kernel-trace summary: bench.py (ResNet-50 conv layers, batch 64: full-width train step + reconfiguration sweep + pruned-width train step)")
    o.append("kernel sources: %s" % bench["config"].get("kernel_sources"))
    o.append("commands (from /tmp, TMPDIR=/tmp):")
    o.append("  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline > <out>/bench.json")
    o.append("  python3 -m paper_1901_09290_amd.profile_report step --stats <out>/..._kernel_stats.csv --bench <out>/bench.json --out <this file>")
    o.append("durations in microseconds; the run holds the timed graph replays of the step plus the per-phase and per-family timing passes of bench.py")
    o.append("")
    o.append("%-66s %7s %11s %9s %9s %9s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "pct"))
    tot, calls = collections.defaultdict(float), collections.defaultdict(int)
    for r in rows:
        n = short(r["Name"])
        f = family(n)
        if f:
            tot[f] += float(r["TotalDurationNs"]) / 1e3
            calls[f] += int(r["Calls"])
        if float(r["Percentage"]) < 0.05:
            continue
        o.append("%-66s %7d %11.1f %9.2f %9.2f %9.2f %6.2f" % (n[:66], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e3,
                 float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    o.append("")
    rl = bench["roofline"]
    o.append("dominant kernel of the step (bench.py 'roofline'): %s" % rl["kernel"])
    if calls["k_igemm_dl"]:
        o.append("  k_igemm_dl (all instantiations): %d launches, %.1f us total, %.2f us average.  Inside the step the input-gradient launches share the"
                 % (calls["k_igemm_dl"], tot["k_igemm_dl"], tot["k_igemm_dl"] / calls["k_igemm_dl"]))
        o.append("  chip with the weight-gradient kernels on the side streams, so this average is above that of the kernel running alone;")
        o.append("  bench.py roofline.avg_launch_ms (HIP events around the family passes, where it runs alone, zero-fill launches of strided layers included): %.2f us" % (rl["avg_launch_ms"] * 1e3))
    if calls["k_wgrad_dl"]:
        o.append("  k_wgrad_dl (all instantiations): %d launches, %.1f us total, %.2f us average; k_wgrad_reduce: %d launches, %.2f us average"
                 % (calls["k_wgrad_dl"], tot["k_wgrad_dl"], tot["k_wgrad_dl"] / calls["k_wgrad_dl"], calls["k_wgrad_reduce"],
                    tot["k_wgrad_reduce"] / max(1, calls["k_wgrad_reduce"])))
    o.append("")
    o.append("bench.py line of the same run (value, step time, roofline):")
    o.append(json.dumps({k: bench[k] for k in ("value", "unit", "ms_per_step", "roofline")}))
    _write(a.out, o)


def _write(path: str, lines: List[str]) -> None:
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(f"wrote {path} ({len(lines)} lines)", file=sys.stderr)


def main(argv=None) -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("layers")
    p.add_argument("--manifest", required=True)
    p.add_argument("--trace", required=True)
    p.add_argument("--fetch")
    p.add_argument("--write")
    p.add_argument("--out", required=True)
    p.set_defaults(fn=cmd_layers)
    p = sub.add_parser("traffic")
    p.add_argument("--manifest", required=True)
    p.add_argument("--fetch", required=True)
    p.add_argument("--write", required=True)
    p.add_argument("--out", required=True)
    p.set_defaults(fn=cmd_traffic)
    p = sub.add_parser("mfma")
    p.add_argument("--manifest", required=True)
    p.add_argument("--trace", required=True)
    p.add_argument("--pmc", required=True)
    p.add_argument("--out", required=True)
    p.set_defaults(fn=cmd_mfma)
    p = sub.add_parser("step")
    p.add_argument("--stats", required=True)
    p.add_argument("--bench", required=True)
    p.add_argument("--out", required=True)
    p.set_defaults(fn=cmd_step)
    a = ap.parse_args(argv)
    a.fn(a)


if __name__ == "__main__":
    main()
