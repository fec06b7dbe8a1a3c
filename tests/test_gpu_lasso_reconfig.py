"""GPU parity: group norms, lasso gradient, zero-group detection, reconciliation, plan and the
compaction gathers through the C ABI against the fp64 oracle (masks/indices/gathers bit-exact)."""
import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import binding as B
from paper_1901_09290_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _norms_gpu(w, pitch=None, shadow=False):
    from gpu_util import DEV, dev_f32, workspace
    K, C = w.shape[0], w.shape[-1]
    RS = w.size // (K * C)
    pitch = pitch or C
    wd = dev_f32(w, pitch)
    on = torch.full((K,), float("nan"), device=DEV)
    inn = torch.full((C,), float("nan"), device=DEV)
    sh = None
    if shadow:
        sh = torch.empty((K, RS, pitch), dtype=torch.bfloat16, device=DEV)
        sh.view(torch.int16).fill_(0x7FC0)
    ws = workspace(B.group_norms_workspace_bytes(K, RS, C))
    B.group_norms(wd, K, RS, C, pitch, on, inn, sh, ws)
    torch.cuda.synchronize()
    return wd, on, inn, sh


NORM_SHAPES = [(16, 3, 3, 16), (64, 1, 1, 64), (256, 1, 1, 64), (64, 7, 7, 3), (128, 3, 3, 128), (37, 3, 3, 51),
               (203, 1, 1, 811), (512, 1, 1, 2048), (5, 1, 1, 1), (1, 1, 1, 9), (700, 3, 3, 24),
               # one, two, four and eight 16-byte columns per thread, rows that do not fill the last batch of a chunk
               (207, 1, 1, 655), (45, 3, 3, 209), (300, 1, 1, 1000), (2100, 1, 1, 260), (3, 1, 1, 2048), (20, 1, 1, 516),
               (4099, 1, 1, 4), (131, 3, 3, 12), (17, 5, 5, 2047)]


@pytest.mark.parametrize("shape", NORM_SHAPES)
@pytest.mark.parametrize("padded", [False, True])
def test_group_norms_and_shadow(shape, padded):
    from gpu_util import F32_TOL, host_bf16, pitch8, rel_err
    rng = np.random.Generator(np.random.PCG64(sum(shape)))
    w = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.05)
    w[0] = 0.0
    w[..., shape[-1] - 1] = 0.0
    pitch = pitch8(shape[-1]) if padded else shape[-1]
    _, on, inn, sh = _norms_gpu(w, pitch, shadow=True)
    ron, rin = oracle.group_norms(w)
    assert rel_err(on.cpu().numpy(), ron) <= F32_TOL
    assert rel_err(inn.cpu().numpy(), rin) <= F32_TOL
    assert on[0].item() == 0.0 and inn[-1].item() == 0.0          # exact zeros stay exact
    # shadow = round-to-nearest-even bf16 of the master weights, bit for bit
    got = sh.view(torch.int16).cpu().numpy().view(np.uint16).reshape(shape[0], -1, pitch)
    want = wl.bf16_bits(wl.to_bf16_grid(w)).reshape(shape[0], -1, shape[-1])
    assert np.array_equal(got[..., : shape[-1]], want)
    if pitch != shape[-1]:
        assert np.all(got[..., shape[-1]:] == 0x7FC0)


@pytest.mark.parametrize("shape", NORM_SHAPES)
@pytest.mark.parametrize("flags", [3, 1, 2])
def test_group_lasso_grad(shape, flags):
    from gpu_util import F32_TOL, dev_f32, pitch8, rel_err
    rng = np.random.Generator(np.random.PCG64(sum(shape) + flags))
    w = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.05)
    w[0] = 0.0
    w[..., 0] = 0.0
    dw0 = rng.standard_normal(shape, dtype=np.float32)
    lam = 1e-3
    K, C = shape[0], shape[-1]
    RS = w.size // (K * C)
    for pitch in (C, pitch8(C)):
        wd, on, inn, _ = _norms_gpu(w, pitch)
        dwd = dev_f32(dw0, pitch)
        B.group_lasso_grad(wd, on, inn, lam, flags, dwd, K, RS, C, pitch)
        torch.cuda.synchronize()
        got = dwd.cpu().numpy()[..., :C]
        ron, rin = oracle.group_norms(w)
        ref = oracle.group_lasso_grad(w, ron, rin, lam, flags, dw0)
        assert rel_err(got, ref) <= F32_TOL
        if flags == 1:
            assert np.array_equal(got[0], dw0[0])                            # zero out-group: dw untouched
    # pure gradient (dw = 0): 1e-5 on the gradient itself
    wd, on, inn, _ = _norms_gpu(w, C)
    dwd = torch.zeros(shape, dtype=torch.float32, device="cuda:0")
    B.group_lasso_grad(wd, on, inn, lam, flags, dwd, K, RS, C, C)
    torch.cuda.synchronize()
    ref = oracle.group_lasso_grad(w, ron, rin, lam, flags, np.zeros(shape))
    assert rel_err(dwd.cpu().numpy(), ref) <= F32_TOL
    g = dwd.cpu().numpy()
    if flags & 1:
        assert np.all(g[0] == 0.0)
    if flags == 2:
        assert np.all(g[..., 0] == 0.0)


def test_batched_norms_and_lasso_match_oracle_per_layer():
    """All layers of a ResNet-32-shaped stack (plus two ragged ones and an unaligned one) through the
    multi-layer calls: more layers than one launch holds, both loader kinds in one call."""
    from gpu_util import DEV, F32_TOL, dev_f32, host_bf16, pitch8, rel_err
    specs, _ = wl.resnet32_layers(N=1)
    shapes = [(s.K, s.R, s.S, s.C) for s in specs] * 2 + [(203, 1, 1, 811), (37, 3, 3, 51), (64, 3, 3, 37)]
    rng = np.random.Generator(np.random.PCG64(21))
    lam = 2e-3
    ws_h, jobs_n, jobs_l, devs = [], [], [], []
    for i, sh in enumerate(shapes):
        w = rng.standard_normal(sh, dtype=np.float32) * np.float32(0.05)
        w[0] = 0.0
        dw0 = rng.standard_normal(sh, dtype=np.float32)
        K, C = sh[0], sh[-1]
        RS = sh[1] * sh[2]
        pitch = C if i == len(shapes) - 1 else pitch8(C)          # the last layer is stored unaligned
        wd, dwd = dev_f32(w, pitch), dev_f32(dw0, pitch)
        on = torch.full((K,), float("nan"), device=DEV)
        inn = torch.full((C,), float("nan"), device=DEV)
        sh_t = torch.zeros((K, RS, pitch), dtype=torch.bfloat16, device=DEV)
        flags = 1 if i == 0 else 3
        jobs_n.append(B.layer_weights(wd, K, RS, C, pitch, on, inn, sh_t))
        jobs_l.append(B.layer_lasso(wd, on, inn, dwd, K, RS, C, pitch, flags))
        ws_h.append((w, dw0, flags))
        devs.append((wd, dwd, on, inn, sh_t))
    assert len(shapes) > 64
    ws = torch.empty(B.group_norms_batched_workspace_bytes(jobs_n), dtype=torch.uint8, device=DEV)
    B.group_norms_batched(jobs_n, ws)
    B.group_lasso_grad_batched(jobs_l, lam)
    torch.cuda.synchronize()
    for (w, dw0, flags), (wd, dwd, on, inn, sh_t), sh in zip(ws_h, devs, shapes):
        ron, rin = oracle.group_norms(w)
        assert rel_err(on.cpu().numpy(), ron) <= F32_TOL and rel_err(inn.cpu().numpy(), rin) <= F32_TOL
        ref = oracle.group_lasso_grad(w, ron, rin, lam, flags, dw0)
        assert rel_err(dwd.cpu().numpy()[..., : sh[-1]], ref) <= F32_TOL
        got = host_bf16(sh_t, sh[-1]).reshape(sh)
        assert np.array_equal(got, wl.to_bf16_grid(w))
    # running the same call again gives bit-identical norms (fixed reduction order)
    before = [d[2].clone() for d in devs]
    B.group_norms_batched(jobs_n, ws)
    torch.cuda.synchronize()
    assert all(torch.equal(a, d[2]) for a, d in zip(before, devs))


def test_zero_groups_bit_exact_and_threshold_edges():
    from gpu_util import DEV
    rng = np.random.Generator(np.random.PCG64(5))
    n = 5000
    norms = np.abs(rng.standard_normal(n)).astype(np.float32) * np.float32(0.1) + np.float32(1e-2)
    norms[rng.choice(n, 1500, replace=False)] = 0.0
    nd = torch.from_numpy(norms).to(DEV)
    for thr in (1e-6, 1e-4, 0.0, -1.0, 0.05):
        z = torch.full((n,), 7, dtype=torch.uint8, device=DEV)
        B.zero_groups(nd, n, thr, z)
        torch.cuda.synchronize()
        ref = oracle.zero_groups(norms.astype(np.float64), float(np.float32(thr)))
        assert np.array_equal(z.cpu().numpy(), ref)
    # exactly at the threshold: strict comparison
    v = np.array([1e-4, np.nextafter(np.float32(1e-4), np.float32(0)), np.nextafter(np.float32(1e-4), np.float32(1))],
                 dtype=np.float32)
    z = torch.zeros(3, dtype=torch.uint8, device=DEV)
    B.zero_groups(torch.from_numpy(v).to(DEV), 3, float(np.float32(1e-4)), z)
    torch.cuda.synchronize()
    assert z.cpu().numpy().tolist() == [0, 1, 0]
    B.zero_groups(nd, 0, 1.0, z)  # empty input is a no-op


def test_norms_to_masks_match_oracle_near_threshold():
    """fp32 GPU norms vs fp64 oracle norms decide the same mask except inside a relative 1e-5 guard
    band around the threshold (the only place where both answers are acceptable)."""
    from gpu_util import DEV
    rng = np.random.Generator(np.random.PCG64(6))
    K, RS, C = 300, 9, 40
    scale = (10.0 ** rng.uniform(-6, -2, size=(K, 1, 1))).astype(np.float32)
    w = (rng.standard_normal((K, RS, C), dtype=np.float32) * scale).astype(np.float32)
    thr = 1e-4
    _, on, inn, _ = _norms_gpu(w.reshape(K, 3, 3, C))
    z = torch.zeros(K, dtype=torch.uint8, device=DEV)
    B.zero_groups(on, K, thr, z)
    torch.cuda.synchronize()
    ron, _ = oracle.group_norms(w)
    ref = oracle.zero_groups(ron, thr)
    safe = np.abs(ron - thr) > 1e-5 * thr
    assert safe.sum() > K - 5 and ref.sum() > 10 and ref.sum() < K - 10
    assert np.array_equal(z.cpu().numpy()[safe], ref[safe])


@pytest.mark.parametrize("n,n_prod,n_cons", [(64, 1, 1), (2048, 4, 5), (37, 7, 0), (1000, 0, 3), (1, 2, 2)])
def test_reconcile_and_plan_bit_exact(n, n_prod, n_cons):
    from gpu_util import DEV
    rng = np.random.Generator(np.random.PCG64(n + n_prod))
    masks = [(rng.random(n) < 0.7).astype(np.uint8) for _ in range(n_prod + n_cons)]
    md = [torch.from_numpy(m).to(DEV) for m in masks]
    keep = torch.full((n,), 9, dtype=torch.uint8, device=DEV)
    B.reconcile_edge(md[:n_prod], md[n_prod:], n, keep)
    idx = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    B.compact_plan(keep, n, idx, cnt)
    torch.cuda.synchronize()
    rkeep = oracle.reconcile_edge(masks[:n_prod], masks[n_prod:])
    ridx = oracle.compact_plan(rkeep)
    assert np.array_equal(keep.cpu().numpy(), rkeep)
    assert cnt.item() == ridx.size
    assert np.array_equal(idx.cpu().numpy()[: ridx.size], ridx)
    assert np.all(idx.cpu().numpy()[ridx.size:] == -1)


@pytest.mark.parametrize("n", [0, 1, 63, 64, 1023, 1024, 1025, 5000])
@pytest.mark.parametrize("mode", ["all", "none", "random"])
def test_plan_edge_cases(n, mode):
    from gpu_util import DEV
    rng = np.random.Generator(np.random.PCG64(n))
    keep = {"all": np.ones(n, np.uint8), "none": np.zeros(n, np.uint8),
            "random": (rng.random(n) < 0.5).astype(np.uint8) * 3}[mode]       # any non-zero byte keeps
    kd = torch.from_numpy(keep).to(DEV) if n else torch.empty(1, dtype=torch.uint8, device=DEV)
    idx = torch.full((max(n, 1),), -1, dtype=torch.int32, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    B.compact_plan(kd, n, idx, cnt)
    torch.cuda.synchronize()
    ridx = oracle.compact_plan(keep)
    assert cnt.item() == ridx.size
    assert np.array_equal(idx.cpu().numpy()[: ridx.size], ridx)


@pytest.mark.parametrize("shape,pad_out", [((16, 3, 3, 16), False), ((203, 1, 1, 811), True), ((64, 7, 7, 3), False),
                                           ((130, 3, 3, 37), True)])
def test_compact_weights_bit_exact(shape, pad_out):
    from gpu_util import DEV, dev_f32, pitch8
    rng = np.random.Generator(np.random.PCG64(sum(shape)))
    K, C = shape[0], shape[-1]
    RS = shape[1] * shape[2]
    w = rng.standard_normal(shape, dtype=np.float32)
    ik = np.sort(rng.choice(K, max(1, K * 2 // 3), replace=False)).astype(np.int32)
    ic = np.sort(rng.choice(C, max(1, C * 3 // 5), replace=False)).astype(np.int32)
    wd = dev_f32(w)
    for use_k, use_c in ((True, True), (True, False), (False, True)):
        Kp, Cp = (ik.size if use_k else K), (ic.size if use_c else C)
        op = pitch8(Cp) if pad_out else Cp
        out = torch.full((Kp, RS, op), float("nan"), dtype=torch.float32, device=DEV)
        B.compact_weights(wd, K, RS, C, C, torch.from_numpy(ik).to(DEV) if use_k else None, Kp,
                          torch.from_numpy(ic).to(DEV) if use_c else None, Cp, out, op)
        torch.cuda.synchronize()
        ref = oracle.compact_weights(w, ik if use_k else None, ic if use_c else None).astype(np.float32)
        got = out.cpu().numpy()
        assert np.array_equal(got[..., :Cp].reshape(ref.shape), ref)
        assert np.all(np.isnan(got[..., Cp:]))


def test_compact_vector_bit_exact():
    from gpu_util import DEV
    rng = np.random.Generator(np.random.PCG64(11))
    n = 2048
    idx = np.sort(rng.choice(n, 1301, replace=False)).astype(np.int32)
    idd = torch.from_numpy(idx).to(DEV)
    for dt in (np.uint8, np.int16, np.float32, np.float64):
        v = (rng.standard_normal(n) * 100).astype(dt)
        out = torch.zeros(idx.size, dtype=getattr(torch, np.dtype(dt).name), device=DEV)
        B.compact_vector(torch.from_numpy(v).to(DEV), np.dtype(dt).itemsize, idd, idx.size, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.compact_vector(v, idx))
    B.compact_vector(idd, 4, idd, 0, idd)  # empty gather is a no-op


@pytest.mark.parametrize("pixels,C,pad", [(4 * 16 * 16, 16, 0), (3 * 7 * 7, 203, 8), (1000, 64, 8),
                                          (129, 811, 8), (50, 5, 0), (1, 8, 0), (77, 45, 24), (1000, 209, 16),
                                          (33, 21, 3), (9, 30, 13)])
def test_compact_nhwc_bit_exact(pixels, C, pad):
    """pad: 0 = dense rows; 8 = pitches rounded up to 8; 16 / 24 = output pitch with whole spare vectors behind the
    last one; other values = output pitch Cp + pad (rows neither aligned nor a multiple of 8).  Padding channels up
    to the next multiple of 8 are written as zero, the rest of the row is left alone."""
    from gpu_util import DEV, pitch8
    rng = np.random.Generator(np.random.PCG64(pixels + C))
    x = rng.integers(0, 65536, size=(pixels, C)).astype(np.uint16)
    idx = np.sort(rng.choice(C, max(1, int(C * 0.6)), replace=False)).astype(np.int32)
    xp = pitch8(C) if pad % 8 == 0 and pad else C
    op = idx.size if pad == 0 else (pitch8(idx.size) + pad - 8 if pad % 8 == 0 else idx.size + pad)
    xfull = np.full((pixels, xp), 0xDEAD, dtype=np.uint16)
    xfull[:, :C] = x
    xd = torch.from_numpy(xfull.view(np.int16)).to(DEV).view(torch.bfloat16)
    out = torch.empty((pixels, op), dtype=torch.bfloat16, device=DEV)
    out.view(torch.int16).fill_(0x1234)
    B.compact_nhwc(xd, pixels, C, xp, torch.from_numpy(idx).to(DEV), idx.size, out, op)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:, : idx.size], oracle.compact_nhwc(x, idx))
    zero_to = min(op, (idx.size + 7) // 8 * 8)
    assert np.all(got[:, idx.size:zero_to] == 0)
    assert np.all(got[:, zero_to:] == 0x1234)


def test_cfg1_reconfiguration_end_to_end():
    """cfg1: norms -> zero masks -> keep -> plan -> compact weights and activations; then the
    compacted layer's forward output equals the kept channels of the full layer's output (GPU vs GPU,
    bit for bit: dropped terms are exact zeros and the survivors are accumulated in the same order
    only if the tiling matches, so compare against the oracle within the conv tolerance instead)."""
    from gpu_util import CONV_TOL, DEV, dev_bf16, host_bf16, rel_err, run_conv_all
    c = wl.cfg1(0)
    spec, w = c["spec"], c["w_master"]
    wd, on, inn, sh = _norms_gpu(w, shadow=True)
    zo = torch.zeros(16, dtype=torch.uint8, device=DEV)
    zi = torch.zeros(16, dtype=torch.uint8, device=DEV)
    B.zero_groups(on, 16, c["thr"], zo)
    B.zero_groups(inn, 16, c["thr"], zi)
    torch.cuda.synchronize()
    assert np.flatnonzero(zo.cpu().numpy()).tolist() == c["zero_out"].tolist()
    assert np.flatnonzero(zi.cpu().numpy()).tolist() == c["zero_in"].tolist()
    keep_k = torch.zeros(16, dtype=torch.uint8, device=DEV)
    keep_c = torch.zeros(16, dtype=torch.uint8, device=DEV)
    B.reconcile_edge([zo], [], 16, keep_k)
    B.reconcile_edge([], [zi], 16, keep_c)
    ik = torch.zeros(16, dtype=torch.int32, device=DEV)
    ic = torch.zeros(16, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, dtype=torch.int32, device=DEV)
    nc = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.compact_plan(keep_k, 16, ik, nk)
    B.compact_plan(keep_c, 16, ic, nc)
    torch.cuda.synchronize()
    assert nk.item() == 12 and nc.item() == 12
    w2 = torch.empty((12, 9, 12), dtype=torch.float32, device=DEV)
    B.compact_weights(wd, 16, 9, 16, 16, ik, 12, ic, 12, w2, 12)
    xd = dev_bf16(c["x"])
    x2 = torch.empty((4, 16, 16, 12), dtype=torch.bfloat16, device=DEV)
    B.compact_nhwc(xd, 4 * 16 * 16, 16, 16, ic, 12, x2, 12)
    torch.cuda.synchronize()
    rik, ric = ik.cpu().numpy()[:12], ic.cpu().numpy()[:12]
    assert np.array_equal(w2.cpu().numpy().reshape(12, 3, 3, 12), oracle.compact_weights(w, rik, ric).astype(np.float32))
    assert np.array_equal(host_bf16(x2), c["x"][..., ric])
    # compacted layer on the GPU vs the oracle's full layer restricted to kept channels
    spec2 = wl.ConvSpec("cfg1c", 4, 16, 16, 12, 12, 3, 3, 1, 1, None, None)
    wc = wl.to_bf16_grid(w2.cpu().numpy().reshape(12, 3, 3, 12))
    y2, dx2, dw2 = run_conv_all(spec2, host_bf16(x2), wc, c["dy"][..., rik])
    s = oracle.shape_of(spec)
    assert rel_err(y2, oracle.conv_fwd(s, c["x"], c["w"])[..., rik]) <= CONV_TOL
    assert rel_err(dx2, oracle.conv_bwd_data(s, c["dy"], c["w"])[..., ric]) <= CONV_TOL
    assert rel_err(dw2, oracle.conv_bwd_weight(s, c["x"], c["dy"])[rik][..., ric]) <= CONV_TOL


def test_multi_job_reconfiguration_equals_single_calls_and_oracle():
    """A small network with a residual-style shared edge, swept once through the multi-job calls and once
    through the single-tensor calls: identical masks, plans and compacted tensors, and both equal the oracle."""
    from paper_1901_09290_amd import harness as hz
    specs = [
        wl.ConvSpec("m0", 2, 12, 12, 3, 300, 3, 3, 1, 1, None, 0, first=True),
        wl.ConvSpec("m1", 2, 12, 12, 300, 37, 1, 1, 1, 0, 0, 1),
        wl.ConvSpec("m2", 2, 12, 12, 37, 300, 3, 3, 1, 1, 1, 0),
        wl.ConvSpec("m3", 2, 12, 12, 300, 1100, 1, 1, 1, 0, 0, 2),
        wl.ConvSpec("m4", 2, 12, 12, 1100, 9, 1, 1, 1, 0, 2, None),
    ]
    edges = [wl.Edge("e0", 300, [0, 2], [1, 3]), wl.Edge("e1", 37, [1], [2]), wl.Edge("e2", 1100, [3], [4])]
    rng = np.random.Generator(np.random.PCG64(77))
    zero_sets = wl.zeroed_channel_sets(edges, 0.35, rng)
    weights = wl.network_weights(specs, edges, zero_sets, rng)
    a = hz.ReconfigModel(specs, edges, weights, seed=8)
    b = hz.ReconfigModel(specs, edges, weights, seed=8)
    a.detect(1e-6)
    a.compact()
    b.detect_per_call(1e-6)
    b.compact(per_call=True)
    torch.cuda.synchronize()
    assert np.array_equal(a.new_counts, b.new_counts)
    assert a.new_counts.tolist() == [e.n - z.size for e, z in zip(edges, zero_sets)]
    for ta, tb in zip(a.keep + a.zo + a.zi + a.w_out + a.mom_out + a.act_out + [v for vs in a.bn_out for v in vs],
                      b.keep + b.zo + b.zi + b.w_out + b.mom_out + b.act_out + [v for vs in b.bn_out for v in vs]):
        assert torch.equal(ta, tb)
    for e in range(len(edges)):
        n = int(a.new_counts[e])
        keep = np.ones(edges[e].n, dtype=np.uint8)
        keep[zero_sets[e]] = 0
        assert np.array_equal(a.keep[e].cpu().numpy(), keep)
        assert np.array_equal(a.idx[e].cpu().numpy()[:n], oracle.compact_plan(keep))
        assert np.array_equal(b.idx[e].cpu().numpy()[:n], oracle.compact_plan(keep))
    for i, s in enumerate(specs):
        ik = oracle.compact_plan(a.keep[s.out_edge].cpu().numpy()) if s.out_edge is not None else None
        ic = oracle.compact_plan(a.keep[s.in_edge].cpu().numpy()) if s.in_edge is not None else None
        Kp = s.K if ik is None else ik.size
        Cp = s.C if ic is None else ic.size
        op = hz.pitch8(Cp)
        got = a.w_out[i].reshape(-1)[: Kp * s.R * s.S * op].reshape(Kp, s.R, s.S, op).cpu().numpy()[..., :Cp]
        assert np.array_equal(got, oracle.compact_weights(weights[i], ik, ic).astype(np.float32))
        if ik is not None:
            for v, o in zip(a.bn[i], a.bn_out[i]):
                assert np.array_equal(o.cpu().numpy()[:Kp], oracle.compact_vector(v.cpu().numpy(), ik))


def test_more_jobs_than_one_launch_holds():
    """A chain of 130 tiny layers: more edges, weight-shaped tensors, per-channel vectors and activations than the job
    tables of one launch hold (64 / 112 / 224 / 64), so every multi-job call splits; results equal the single calls."""
    from paper_1901_09290_amd import harness as hz
    rng = np.random.Generator(np.random.PCG64(91))
    n_layers = 130
    widths = [int(rng.integers(9, 41)) for _ in range(n_layers)]
    specs, edges = [], []
    c_in = 3
    for i, k in enumerate(widths):
        specs.append(wl.ConvSpec(f"c{i}", 1, 5, 5, c_in, k, 1, 1, 1, 0, None if i == 0 else i - 1,
                                 i if i + 1 < n_layers else None, first=(i == 0)))
        if i + 1 < n_layers:
            edges.append(wl.Edge(f"e{i}", k, [i], [i + 1]))
        c_in = k
    zero_sets = wl.zeroed_channel_sets(edges, 0.3, rng)
    weights = wl.network_weights(specs, edges, zero_sets, rng)
    a = hz.ReconfigModel(specs, edges, weights, seed=5)
    b = hz.ReconfigModel(specs, edges, weights, seed=5)
    a.detect(1e-6)
    a.compact()
    b.detect_per_call(1e-6)
    b.compact(per_call=True)
    torch.cuda.synchronize()
    assert a.new_counts.tolist() == [e.n - z.size for e, z in zip(edges, zero_sets)]
    assert np.array_equal(a.new_counts, b.new_counts)
    for ta, tb in zip(a.keep + a.idx + a.zo + a.zi + a.w_out + a.mom_out + a.act_out + [v for vs in a.bn_out for v in vs],
                      b.keep + b.idx + b.zo + b.zi + b.w_out + b.mom_out + b.act_out + [v for vs in b.bn_out for v in vs]):
        assert torch.equal(ta, tb)
    for i in (0, 63, 64, 111, 112, 129):      # layers on either side of the table boundaries, against the oracle
        s = specs[i]
        ik = oracle.compact_plan(a.keep[s.out_edge].cpu().numpy()) if s.out_edge is not None else None
        ic = oracle.compact_plan(a.keep[s.in_edge].cpu().numpy()) if s.in_edge is not None else None
        Kp = s.K if ik is None else ik.size
        Cp = s.C if ic is None else ic.size
        op = hz.pitch8(Cp)
        got = a.w_out[i].reshape(-1)[: Kp * op].reshape(Kp, 1, 1, op).cpu().numpy()[..., :Cp]
        assert np.array_equal(got, oracle.compact_weights(weights[i], ik, ic).astype(np.float32))


def test_regulariser_value_matches_oracle_and_is_deterministic():
    """GroupLassoReg over a whole network (ResNet-32 shapes + a 100-layer stack that needs two launches):
    device fp64 sum of the device's fp32 norms vs the oracle's fp64 sum of fp64 norms, 1e-5 relative; exact
    against the fp64 sum of the device's own norms; identical on a second run; first-layer exemption honoured."""
    from gpu_util import DEV, F32_TOL
    specs, _ = wl.resnet32_layers(N=2)
    specs = list(specs) + [wl.ConvSpec(f"x{i}", 1, 4, 4, 5 + i % 7, 3 + i % 11, 1, 1, 1, 0, None, None) for i in range(100)]
    rng = np.random.Generator(np.random.PCG64(91))
    jobs, ref_layers, dev_sum, keep = [], [], 0.0, []
    for i, s in enumerate(specs):
        w = wl.master_weights(s, rng)
        flags = 1 if s.first else 3
        wd, on, inn, _ = _norms_gpu(w, shadow=False)
        keep += [wd, on, inn]
        jobs.append(B.layer_penalty(on, inn, s.K, s.C, flags))
        a, b = oracle.group_norms(w)
        ref_layers.append((a, b, flags))
        dev_sum += float(on.double().sum()) + (float(inn.double().sum()) if flags & 2 else 0.0)
    out = torch.full((1,), float("nan"), dtype=torch.float64, device=DEV)
    B.group_lasso_penalty_batched(jobs, out)
    torch.cuda.synchronize()
    got = out.item()
    ref = oracle.group_lasso_penalty(ref_layers)
    assert abs(got - ref) <= F32_TOL * ref
    assert abs(got - dev_sum) <= 1e-12 * ref          # the reduction itself is fp64
    out2 = torch.zeros(1, dtype=torch.float64, device=DEV)
    B.group_lasso_penalty_batched(jobs, out2)
    torch.cuda.synchronize()
    assert out2.item() == got
    B.group_lasso_penalty_batched([], out2)            # no layers: the value is 0
    torch.cuda.synchronize()
    assert out2.item() == 0.0
    # the coefficient that makes the regulariser 25 % of the total loss at a classification loss of 6.9
    lam = B.lasso_set_coeff(6.9, got, 0.25)
    assert abs(lam * got / (6.9 + lam * got) - 0.25) < 1e-12


@pytest.mark.parametrize("pixels,C,pad", [(4 * 16 * 16, 16, False), (3 * 7 * 7, 203, True), (1000, 64, True),
                                          (129, 811, True), (50, 5, False), (1, 8, False), (70000, 72, True)])
def test_scatter_nhwc_bit_exact_and_inverts_the_gather(pixels, C, pad):
    from gpu_util import DEV, pitch8
    rng = np.random.Generator(np.random.PCG64(5000 + pixels + C))
    idx = np.sort(rng.choice(C, max(1, int(C * 0.6)), replace=False)).astype(np.int32)
    Cp = idx.size
    x = rng.integers(1, 65536, size=(pixels, Cp)).astype(np.uint16)
    xp = pitch8(Cp) if pad else Cp
    op = pitch8(C) if pad else C
    xfull = np.full((pixels, xp), 0xDEAD, dtype=np.uint16)
    xfull[:, :Cp] = x
    xd = torch.from_numpy(xfull.view(np.int16)).to(DEV).view(torch.bfloat16)
    idd = torch.from_numpy(idx).to(DEV)
    out = torch.empty((pixels, op), dtype=torch.bfloat16, device=DEV)
    out.view(torch.int16).fill_(0x1234)
    B.scatter_nhwc(xd, pixels, Cp, xp, idd, C, out, op)
    back = torch.empty((pixels, xp), dtype=torch.bfloat16, device=DEV)
    back.view(torch.int16).fill_(0x4321)
    B.compact_nhwc(out, pixels, C, op, idd, Cp, back, xp)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:, :C], oracle.scatter_nhwc(x, idx, C))
    assert np.all(got[:, C:] == 0x1234)                                     # pitch padding untouched
    assert np.array_equal(back.view(torch.int16).cpu().numpy().view(np.uint16)[:, :Cp], x)


@pytest.mark.parametrize("shape,pad", [((16, 3, 3, 16), False), ((40, 1, 1, 203), True), ((7, 7, 7, 3), False),
                                       ((300, 3, 3, 37), True), ((5, 1, 1, 2048), False)])
def test_group_maxabs_is_exact(shape, pad):
    from gpu_util import DEV, dev_f32, pitch8
    rng = np.random.Generator(np.random.PCG64(6000 + sum(shape)))
    w = rng.standard_normal(shape).astype(np.float32)
    w[1] = 0.0
    w[..., 0] = 0.0
    K, C = shape[0], shape[-1]
    RS = shape[1] * shape[2]
    pitch = pitch8(C) if pad else C
    wd = dev_f32(w, pitch)                      # padding is NaN: it must not enter the maxima
    om = torch.full((K,), float("nan"), device=DEV)
    im = torch.full((C,), float("nan"), device=DEV)
    B.group_maxabs(wd, K, RS, C, pitch, om, im)
    torch.cuda.synchronize()
    rom, rim = oracle.group_maxabs(w)
    assert np.array_equal(om.cpu().numpy(), rom.astype(np.float32))          # fp32 maxima of fp32 data: exact
    assert np.array_equal(im.cpu().numpy(), rim.astype(np.float32))
    z = torch.zeros(K, dtype=torch.uint8, device=DEV)
    B.zero_groups(om, K, 1e-4, z)
    torch.cuda.synchronize()
    assert np.array_equal(z.cpu().numpy(), oracle.zero_groups(rom, 1e-4))


def test_apply_zero_bit_exact():
    from gpu_util import DEV, dev_f32, pitch8
    rng = np.random.Generator(np.random.PCG64(7001))
    for shape, pad in (((12, 3, 3, 10), True), ((5, 1, 1, 64), False), ((33, 2, 2, 7), False)):
        w = rng.standard_normal(shape).astype(np.float32)
        K, C = shape[0], shape[-1]
        RS = shape[1] * shape[2]
        zo = (rng.random(K) < 0.3).astype(np.uint8)
        zi = (rng.random(C) < 0.3).astype(np.uint8)
        pitch = pitch8(C) if pad else C
        for mo, mi in ((zo, zi), (None, zi), (zo, None)):
            wd = dev_f32(w, pitch)
            B.apply_zero(wd, K, RS, C, pitch, None if mo is None else torch.from_numpy(mo).to(DEV),
                         None if mi is None else torch.from_numpy(mi).to(DEV))
            torch.cuda.synchronize()
            got = wd.cpu().numpy()
            assert np.array_equal(got[..., :C], oracle.apply_zero(w, mo, mi).astype(np.float32))
            if pitch != C:
                assert np.isnan(got[..., C:]).all()                            # padding untouched


def test_optimizer_step_matches_oracle():
    """One launch updates several layers (vector and element-wise loaders, padded pitches, first-layer
    exemption): weights and momentum against the fp64 oracle at 1e-5; dw and pitch padding untouched; a second
    step from the device's own state also matches (momentum carries over)."""
    from gpu_util import DEV, F32_TOL, dev_f32, pitch8, rel_err
    rng = np.random.Generator(np.random.PCG64(8100))
    shapes = [((16, 3, 3, 3), False, 1), ((40, 1, 1, 203), True, 3), ((64, 3, 3, 64), True, 3), ((7, 5, 5, 11), False, 3),
              ((300, 1, 1, 37), True, 2)]
    lam, lr, mu, wd = 1e-3, 0.1, 0.9, 1e-4
    state = []
    for shape, pad, flags in shapes:
        K, C = shape[0], shape[-1]
        RS = shape[1] * shape[2]
        w = (rng.standard_normal(shape) * 0.1).astype(np.float32)
        w[0] = 0.0                                   # an exactly zero filter
        dw = (rng.standard_normal(shape) * 0.01).astype(np.float32)
        dw[0] = 0.0
        m = (rng.standard_normal(shape) * 0.01).astype(np.float32)
        m[0] = 0.0
        pitch = pitch8(C) if pad else C
        wd_, on, inn, _ = _norms_gpu(w, pitch if pad else None, shadow=False)
        state.append(dict(shape=shape, K=K, RS=RS, C=C, pitch=pitch, flags=flags, w=w, dw=dw, m=m,
                          wd=wd_, dwd=dev_f32(dw, pitch), md=dev_f32(m, pitch), on=on, inn=inn))
    for step in range(2):
        jobs = [B.layer_update(s["wd"], s["dwd"], s["md"], s["on"], s["inn"], s["K"], s["RS"], s["C"], s["pitch"],
                               s["flags"]) for s in state]
        B.sgd_momentum_lasso_batched(jobs, lam, lr, mu, wd)
        torch.cuda.synchronize()
        for s in state:
            on64, in64 = oracle.group_norms(s["w"])
            w_ref, m_ref = oracle.sgd_momentum_lasso(s["w"], s["dw"], s["m"], on64, in64, lam, lr, mu, wd, s["flags"])
            gw, gm = s["wd"].cpu().numpy(), s["md"].cpu().numpy()
            C = s["C"]
            assert rel_err(gw[..., :C], w_ref) <= F32_TOL and rel_err(gm[..., :C], m_ref) <= F32_TOL, s["shape"]
            assert not gw[0, ..., :C].any() and not gm[0, ..., :C].any()          # the zero filter stays exactly zero
            assert np.array_equal(s["dwd"].cpu().numpy()[..., :C], s["dw"])       # the loss gradient is read-only
            if s["pitch"] != C:
                assert np.isnan(gw[..., C:]).all() and np.isnan(gm[..., C:]).all()
            # next step starts from the device's fp32 state and fresh norms of it
            s["w"], s["m"] = gw[..., :C].copy(), gm[..., :C].copy()
            ws = workspace_for(s)
            B.group_norms(s["wd"], s["K"], s["RS"], C, s["pitch"], s["on"], s["inn"], None, ws)
        torch.cuda.synchronize()


def workspace_for(s):
    from gpu_util import workspace
    return workspace(B.group_norms_workspace_bytes(s["K"], s["RS"], s["C"]))


def test_norms_with_zero_masks_in_one_call():
    """pt_group_norms_detect_batched: norms bit-identical to pt_group_norms_batched's, masks bit-identical to
    pt_zero_groups on those norms and to the oracle's (groups are exactly zero or far above the threshold), at
    several thresholds including the ones that mark nothing."""
    from gpu_util import DEV, dev_f32, pitch8
    rng = np.random.Generator(np.random.PCG64(77))
    shapes = [(64, 3, 3, 64), (203, 1, 1, 811), (37, 3, 3, 51), (655, 1, 1, 207), (16, 7, 7, 3), (64, 3, 3, 37)]
    host, devs = [], []
    for i, sh in enumerate(shapes):
        w = rng.standard_normal(sh, dtype=np.float32) * np.float32(0.05)
        K, C = sh[0], sh[-1]
        zo = rng.choice(K, max(1, K // 3), replace=False)
        zi = rng.choice(C, max(1, C // 4), replace=False)
        w = wl.zero_groups_in_weights(w, zo, zi)
        pitch = C if i == len(shapes) - 1 else pitch8(C)          # the last layer is stored unaligned
        t = dict(w=dev_f32(w, pitch), K=K, RS=sh[1] * sh[2], C=C, pitch=pitch)
        for name, n, dt in (("on", K, torch.float32), ("inn", C, torch.float32), ("on2", K, torch.float32),
                            ("inn2", C, torch.float32), ("zo", K, torch.uint8), ("zi", C, torch.uint8),
                            ("zo2", K, torch.uint8), ("zi2", C, torch.uint8)):
            t[name] = torch.full((n,), 7, dtype=dt, device=DEV)
        host.append(w)
        devs.append(t)
    jobs_d = [B.layer_detect(t["w"], t["K"], t["RS"], t["C"], t["pitch"], t["on"], t["inn"], t["zo"], t["zi"]) for t in devs]
    jobs_n = [B.layer_weights(t["w"], t["K"], t["RS"], t["C"], t["pitch"], t["on2"], t["inn2"], None) for t in devs]
    ws = torch.empty(B.group_norms_detect_batched_workspace_bytes(jobs_d), dtype=torch.uint8, device=DEV)
    assert ws.numel() == B.group_norms_batched_workspace_bytes(jobs_n)
    B.group_norms_batched(jobs_n, ws)
    for thr in (1e-6, 1e-4, 0.0, -1.0, 1e9):
        B.group_norms_detect_batched(jobs_d, thr, ws)
        for t in devs:
            B.zero_groups(t["on2"], t["K"], thr, t["zo2"])
            B.zero_groups(t["inn2"], t["C"], thr, t["zi2"])
        torch.cuda.synchronize()
        for w, t in zip(host, devs):
            assert torch.equal(t["on"], t["on2"]) and torch.equal(t["inn"], t["inn2"])
            assert torch.equal(t["zo"], t["zo2"]) and torch.equal(t["zi"], t["zi2"])
            ron, rin = oracle.group_norms(w)
            assert np.array_equal(t["zo"].cpu().numpy(), oracle.zero_groups(ron.astype(np.float32), thr))
            assert np.array_equal(t["zi"].cpu().numpy(), oracle.zero_groups(rin.astype(np.float32), thr))
            if 0.0 < thr < 1.0:
                assert int(t["zo"].sum()) == max(1, t["K"] // 3) and int(t["zi"].sum()) == max(1, t["C"] // 4)
