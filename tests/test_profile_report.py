"""Host logic of the profiler-summary writer: splitting a kernel trace into calls by marker kernels, scaling the
byte counters by the copy probe, and the figures derived from them (no GPU, synthetic csv files)."""
import csv
import json
import os

import pytest

from paper_1901_09290_amd import profile_report as pr

MARK = "pt::k_zero_groups(float const*, int, float, unsigned char*)"
IGEMM = "void pt::k_igemm_dl<128, 64, 4, 2, 3, false, false, false, true>(pt::IgemmArgs)"
WGRAD = "void pt::k_wgrad_dl<128, 128, 64, 2, 2, 3, 1, 1, 2>(pt::WgradArgs)"
REDUCE = "void pt::k_wgrad_reduce4<true>(float const*, int)"
PROBE = "void at::native::vectorized_elementwise_kernel<4, at::native::neg_kernel_cuda(at::TensorIteratorBase&)::{lambda()#1}>(int)"


def _manifest(tmp_path):
    calls = []
    for net in ("full", "pruned", "pruned_up64"):
        calls += [
            {"net": net, "kind": "fwd", "layer": "a", "shape": [64, 56, 56, 64, 64, 1, 1, 1, 0], "flops": 2 * 10**9, "bytes": 8 * 10**7},
            {"net": net, "kind": "bwd_data", "layer": "a", "shape": [64, 56, 56, 64, 64, 1, 1, 1, 0], "flops": 25 * 10**9, "bytes": 4 * 10**7},
            {"net": net, "kind": "bwd_weight_lasso", "layer": "a", "shape": [64, 56, 56, 64, 64, 1, 1, 1, 0], "flops": 2 * 10**9, "bytes": 8 * 10**7},
        ]
    man = {"batch": 64, "marker": "k_zero_groups", "nets": ["full", "pruned", "pruned_up64"], "calls": calls,
           "kernel_sources": "0123456789abcdef", "peak_bf16_tflops": 2500.0, "peak_hbm_GBps": 8000.0,
           "copy_probe": {"read_bytes": 1 << 30, "write_bytes": 1 << 30}}
    p = tmp_path / "manifest.json"
    p.write_text(json.dumps(man))
    return man, str(p)


def _dispatches(scale=1.0):
    """Launch order of a layer pass: per network, untimed first launches, three markers, then call + marker."""
    seq = []
    for net_i in range(3):
        seq += [(IGEMM, 50), (IGEMM, 50), (WGRAD, 50)]                       # first launches, before the triple
        seq += [(MARK, 2)] * 3
        seq += [(IGEMM, 20 * scale), (MARK, 2)]                              # fwd: one kernel
        seq += [(IGEMM, 5), (IGEMM, 5), (IGEMM, 5), (IGEMM, 5), (MARK, 2)]   # strided bwd_data: four classes
        seq += [(WGRAD, 30), (REDUCE, 4), (MARK, 2)]                         # bwd_weight: main + reduction
    seq += [(PROBE, 300)] * 3
    return seq


def _write_trace(path, seq):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Kind", "Dispatch_Id", "Kernel_Name", "Start_Timestamp", "End_Timestamp"])
        t = 1000
        for i, (name, us) in enumerate(seq):
            w.writerow(["KERNEL_DISPATCH", i + 1, name, t, t + int(us * 1000)])
            t += int(us * 1000) + 3000


def _write_counters(path, seq, counter, value_of):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (name, _us) in enumerate(seq):
            w.writerow([i + 1, name, counter, value_of(name)])


def test_trace_splits_into_the_manifests_calls(tmp_path):
    man, _ = _manifest(tmp_path)
    t = str(tmp_path / "t.csv")
    _write_trace(t, _dispatches())
    segs = pr.split_calls(pr.load_trace(t), man)
    assert [len(s) for s in segs] == [1, 4, 2] * 3
    assert all(pr.family(r["name"]) == "k_igemm_dl" for r in segs[1])
    assert [pr.family(r["name"]) for r in segs[2]] == ["k_wgrad_dl", "k_wgrad_reduce"]


def test_missing_marker_triple_is_an_error(tmp_path):
    man, _ = _manifest(tmp_path)
    t = str(tmp_path / "t.csv")
    _write_trace(t, _dispatches()[:20])
    with pytest.raises(SystemExit):
        pr.split_calls(pr.load_trace(t), man)


def test_layer_table_figures(tmp_path):
    man, mp = _manifest(tmp_path)
    t, out = str(tmp_path / "t.csv"), str(tmp_path / "layers.txt")
    _write_trace(t, _dispatches())
    pr.main(["layers", "--manifest", mp, "--trace", t, "--out", out])
    text = open(out).read()
    assert "kernel sources: 0123456789abcdef" in text
    row = [l for l in text.splitlines() if l.startswith("a ")][0]
    fwd, bwd, wgrad = [c.split() for c in row.split("|")[1:]]
    # fwd: 2 GF and 80 MB in 20 us -> 100 TFLOP/s, 4000 GB/s; roof = 80 MB / 8 TB/s = 10 us (hbm), frac 0.5
    assert [float(v) for v in fwd[:4]] == [20.0, 100.0, 4000.0, 0.5] and fwd[4] == "h"
    # bwd_data: 25 GF in 4 x 5 us; roof = 25 GF / 2.5 PFLOP/s = 10 us (mfma)
    assert float(bwd[0]) == 20.0 and float(bwd[3]) == 0.5 and bwd[4] == "m"
    # weight gradient: main kernel 30 us + reduction 4 us
    assert float(wgrad[0]) == 34.0
    assert "total fwd" in text and "2 calls" not in text


def test_traffic_is_scaled_by_the_copy_probe_and_read_back(tmp_path):
    man, mp = _manifest(tmp_path)
    seq = _dispatches()
    f, w, out = str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), str(tmp_path / pr.TRAFFIC_FILE)
    # the probe reads 2^30 bytes and shows 2^19 units: 2048 bytes per unit of FETCH_SIZE; WRITE_SIZE 1024 bytes per unit
    _write_counters(f, seq, "FETCH_SIZE", lambda n: (1 << 19) if "neg_kernel" in n else (10000 if "igemm" in n else 30000))
    _write_counters(w, seq, "WRITE_SIZE", lambda n: (1 << 20) if "neg_kernel" in n else 5000)
    pr.main(["traffic", "--manifest", mp, "--fetch", f, "--write", w, "--out", out])
    got = pr.read_traffic(out, "igemm")
    assert got["digest"] == "0123456789abcdef"
    # per k_igemm_dl launch: 10000 * 2048 + 5000 * 1024 bytes
    assert got["bytes_per_launch"] == pytest.approx(10000 * 2048 + 5000 * 1024, rel=1e-3)
    got = pr.read_traffic(out, "wgrad")
    # per call: main kernel + reduction pass, each 30000 fetch units and 5000 write units
    assert got["bytes_per_launch"] == pytest.approx(2 * (30000 * 2048 + 5000 * 1024), rel=1e-3)
    assert pr.read_traffic(str(tmp_path / "absent.txt"), "igemm") is None


def test_mfma_summary(tmp_path):
    man, mp = _manifest(tmp_path)
    seq = _dispatches()
    t, p, out = str(tmp_path / "t.csv"), str(tmp_path / "p.csv"), str(tmp_path / "m.txt")
    _write_trace(t, seq)
    # every igemm launch executes 2 GF on the matrix cores: 2e9 / 512 units
    _write_counters(p, seq, "SQ_INSTS_VALU_MFMA_MOPS_BF16", lambda n: 2e9 / 512 if "igemm" in n else 0)
    pr.main(["mfma", "--manifest", mp, "--trace", t, "--pmc", p, "--out", out])
    line = [l for l in open(out).read().splitlines() if l.startswith("full") and "k_igemm_dl<" in l][0]
    cols = line.split()
    # full width: 5 launches (1 fwd of 20 us + 4 bwd_data of 5 us) = 40 us for 10 GF executed -> 250 TFLOP/s = 10% of peak
    assert "250" in cols and "10.0" in cols


def test_source_digest_is_stable_and_names_the_kernel_sources():
    d = pr.source_digest()
    assert len(d) == 16 and d == pr.source_digest()
    assert os.path.isdir(os.path.join(os.path.dirname(pr.__file__), "csrc"))
