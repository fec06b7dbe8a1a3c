"""GPU parity at the benchmark's full sizes and in its launch configuration (channel pitch = next
multiple of 8, buffers built by the harness, multi-layer norm/lasso launches), on outputs the
oracle evaluates one by one; plus the reconfiguration chain on whole networks (bit-exact) and the
HIP-graph replay check.

  cfg3  ResNet-50 conv layers, batch 64, 224x224          sampled y / dx / dw of every distinct shape
  cfg4  the same network at ragged pruned widths (seed 3)  sampled y / dx / dw of every distinct shape
  cfg2  ResNet-32 (CIFAR), batch 128                       reconfiguration chain, residual-stage union
  cfg5  ResNet-50 reconfiguration sweep, seeds 10..14      masks, plans, gathers bit-exact
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1901_09290_amd import binding as B
from paper_1901_09290_amd import workloads as wl

pytestmark = pytest.mark.gpu

N_RANDOM = 4000        # random elements per tensor, on top of the corners and of one element per tile block
LAMBDA_VISIBLE = 1e3   # makes the regulariser's term comparable to the data gradient (|w| ~ 0.05, |dw| ~ 10^2)


def _corner_and_random(shape, n, rng):
    """Flat indices: the extreme corners of the tensor (borders, first/last channel) + n random ones."""
    total = int(np.prod(shape))
    corners = []
    for pick in np.ndindex(*(2,) * len(shape)):
        corners.append(np.ravel_multi_index([(d - 1) * p for d, p in zip(shape, pick)], shape))
    idx = np.concatenate([np.array(corners, dtype=np.int64), wl.sample_indices(total, n, rng)])
    return np.unique(idx)


def _block_samples(rows, cols, rng, rb=64, cb=32):
    """One random element in every rb x cb block of a [rows, cols] matrix, as flat indices: every output tile of
    every launch (tiles are multiples of 64 rows and 32 columns) is seen, its ragged last ones included."""
    r0 = np.arange(0, rows, rb, dtype=np.int64)
    c0 = np.arange(0, cols, cb, dtype=np.int64)
    R, Cc = np.meshgrid(r0, c0, indexing="ij")
    r = R + (rng.random(R.shape) * np.minimum(rb, rows - R)).astype(np.int64)
    c = Cc + (rng.random(Cc.shape) * np.minimum(cb, cols - Cc)).astype(np.int64)
    return (r * cols + c).reshape(-1)


def _samples(shape, rows, cols, rng):
    return np.unique(np.concatenate([_corner_and_random(shape, N_RANDOM, rng), _block_samples(rows, cols, rng)]))


def _sampled_err(got, ref):
    """The conv tolerance metric on a sample: rms is taken over the sampled reference values."""
    from gpu_util import rel_err
    return rel_err(got, ref)


def _run_layer_as_the_step_does(spec, t, lam):
    """One layer through the calls Network.train_step makes for it: norms (+ bf16 weights), forward, the k-innermost
    filter copy and the workspace-free input gradient, and the weight gradient with the regulariser folded in."""
    from paper_1901_09290_amd import harness as hz
    layer = hz.ConvLayer(spec, host=t)
    ws = hz.make_workspace([layer])
    layer.norms(ws)
    layer.fwd(ws)
    if layer.w_crsk is not None:
        B.weights_to_crsk_batched([B.layer_crsk(layer.w_bf16, layer.w_crsk, spec.K, layer.RS, spec.C, layer.wp)])
        layer.bwd_data_crsk()
    layer.bwd_weight_lasso(ws, lam)
    torch.cuda.synchronize()
    return layer


def _lasso_term(t, spec, layer, lam):
    ron, rin = oracle.group_norms(t["w"])
    return oracle.group_lasso_grad(t["w"], ron, rin, lam, layer.lasso_flags, np.zeros((spec.K, spec.R, spec.S, spec.C)))


def _check_padding_stays_zero(layer, spec):
    # pitch padding of the outputs stays zero (the harness allocates zero-filled buffers)
    if layer.yp != spec.K:
        assert not bool(layer.y[..., spec.K:].any())
    if layer.wp != spec.C:
        assert not bool(layer.dw[..., spec.C:].any())
    if layer.dx is not None and layer.xp != spec.C:
        assert not bool(layer.dx[..., spec.C:].any())


def _check_layer_sampled(spec, seed):
    from gpu_util import CONV_TOL, host_bf16
    rng = np.random.Generator(np.random.PCG64(seed))
    t = wl.conv_tensors(spec, rng)
    layer = _run_layer_as_the_step_does(spec, t, LAMBDA_VISIBLE)
    s = oracle.shape_of(spec)
    # the shadow copy is the exact bf16 image of the master weights (already on the bf16 grid)
    assert np.array_equal(host_bf16(layer.w_bf16, spec.C), t["w"])
    y = host_bf16(layer.y, spec.K).reshape(-1)
    iy = _samples((spec.N, spec.P, spec.Q, spec.K), spec.N * spec.P * spec.Q, spec.K, rng)
    assert _sampled_err(y[iy], oracle.conv_fwd_at(s, t["x"], t["w"], iy)) <= CONV_TOL, spec
    if layer.dx is not None:
        dx = host_bf16(layer.dx, spec.C).reshape(-1)
        ix = _samples((spec.N, spec.H, spec.W, spec.C), spec.N * spec.H * spec.W, spec.C, rng)
        assert _sampled_err(dx[ix], oracle.conv_bwd_data_at(s, t["dy"], t["w"], ix)) <= CONV_TOL, spec
    dw = layer.dw.cpu().numpy()[..., : spec.C].reshape(-1)
    iw = _samples((spec.K, spec.R, spec.S, spec.C), spec.K, spec.R * spec.S * spec.C, rng)
    ref = oracle.conv_bwd_weight_at(s, t["x"], t["dy"], iw) + _lasso_term(t, spec, layer, LAMBDA_VISIBLE).reshape(-1)[iw]
    assert _sampled_err(dw[iw], ref) <= CONV_TOL, spec
    _check_padding_stays_zero(layer, spec)


def _check_layer_whole(spec, seed):
    """Whole tensors of one layer, run as the step runs it, against the oracle."""
    from gpu_util import CONV_TOL, host_bf16, rel_err
    rng = np.random.Generator(np.random.PCG64(seed))
    t = wl.conv_tensors(spec, rng)
    layer = _run_layer_as_the_step_does(spec, t, LAMBDA_VISIBLE)
    s = oracle.shape_of(spec)
    assert rel_err(host_bf16(layer.y, spec.K), oracle.conv_fwd(s, t["x"], t["w"])) <= CONV_TOL, spec
    if layer.dx is not None:
        assert rel_err(host_bf16(layer.dx, spec.C), oracle.conv_bwd_data(s, t["dy"], t["w"])) <= CONV_TOL, spec
    ref = oracle.conv_bwd_weight(s, t["x"], t["dy"]) + _lasso_term(t, spec, layer, LAMBDA_VISIBLE)
    assert rel_err(layer.dw.cpu().numpy()[..., : spec.C], ref) <= CONV_TOL, spec
    _check_padding_stays_zero(layer, spec)


def _cfg3_shapes():
    specs, _ = wl.resnet50_layers(N=64)
    return [s for s, _ in wl.distinct_shapes(specs)]


def _cfg4_shapes():
    specs, edges = wl.resnet50_layers(N=64)
    keep = wl.pruned_keep_sets(edges, seed=3)
    pruned, _ = wl.with_widths(specs, edges, [k.size for k in keep])
    return [s for s, _ in wl.distinct_shapes(pruned)]


@pytest.mark.parametrize("i", range(len(_cfg3_shapes())))
def test_cfg3_resnet50_batch64_sampled(i):
    _check_layer_sampled(_cfg3_shapes()[i], seed=2000 + i)


@pytest.mark.parametrize("i", range(len(_cfg4_shapes())))
def test_cfg4_pruned_ragged_widths_batch64_sampled(i):
    _check_layer_sampled(_cfg4_shapes()[i], seed=3000 + i)


def _at_batch(spec, N):
    import dataclasses
    return dataclasses.replace(spec, N=N)


def test_cfg3_resnet50_shapes_batch2_whole_tensors():
    """Every distinct full-width layer shape at batch 2: whole y / dx / dw, no sampling."""
    for i, spec in enumerate(_cfg3_shapes()):
        _check_layer_whole(_at_batch(spec, 2), seed=2500 + i)


def test_cfg4_pruned_shapes_batch2_whole_tensors():
    for i, spec in enumerate(_cfg4_shapes()):
        _check_layer_whole(_at_batch(spec, 2), seed=3500 + i)


@pytest.mark.parametrize("norms_head,branches", [(11, True), (None, True), (None, False)],
                         ids=["norms_split_over_two_streams", "norms_before_forward", "shortcuts_on_the_main_stream"])
def test_cfg2_resnet32_train_step_on_side_streams_against_oracle(norms_head, branches, monkeypatch):
    """Network.train_step as the benchmark runs it (norms split over two streams or all ahead of the forward pass,
    k-innermost filter copies, the input gradients of the blocks' shortcut convolutions on a side stream or in line, weight
    gradients with the regulariser folded in on four side streams, zero padding vouched for) on the whole ResNet-32
    stack at batch 128: every layer's norms, y, dx and dw against the oracle.  Then the weights change (one optimizer
    step) and a second step must see the new weights everywhere, the k-innermost copies of the first layers too."""
    from gpu_util import CONV_TOL, F32_TOL, host_bf16, rel_err
    from paper_1901_09290_amd import harness as hz
    specs, _ = wl.resnet32_layers(N=128)
    rng = np.random.Generator(np.random.PCG64(1))
    host = [wl.conv_tensors(s, rng) for s in specs]
    if norms_head is not None:
        monkeypatch.setattr(hz, "NORMS_HEAD_LAYERS", norms_head)
    net = hz.Network([hz.ConvLayer(s, host=t) for s, t in zip(specs, host)])
    assert net.overlap_wgrad and net.fuse_lasso and (net.norm_jobs_tail is not None) == (norms_head is not None)
    # the two stride-2 stages have a shortcut convolution each, forking where their first block starts
    names = [s.name for s in specs]
    assert net.overlap_branches and {names[j]: names[i] for j, i in net.fork.items()} == {
        "stage2_b0_a": "stage2_proj", "stage3_b0_a": "stage3_proj"}
    net.overlap_branches = net.batch_branches_fwd = branches   # (forward: shortcut and first convolution in one call)
    lam = 50.0

    def check(weights):
        for l, t, w in zip(net.layers, host, weights):
            s, o = l.spec, oracle.shape_of(l.spec)
            wb = wl.to_bf16_grid(w)
            ron, rin = oracle.group_norms(w)
            assert rel_err(l.out_norm.cpu().numpy(), ron) <= F32_TOL and rel_err(l.in_norm.cpu().numpy(), rin) <= F32_TOL
            assert np.array_equal(host_bf16(l.w_bf16, s.C), wb)
            assert rel_err(host_bf16(l.y, s.K), oracle.conv_fwd(o, t["x"], wb)) <= CONV_TOL, s
            if l.dx is not None:
                assert rel_err(host_bf16(l.dx, s.C), oracle.conv_bwd_data(o, t["dy"], wb)) <= CONV_TOL, s
            ref = oracle.group_lasso_grad(w, ron, rin, lam, l.lasso_flags, oracle.conv_bwd_weight(o, t["x"], t["dy"]))
            assert rel_err(l.dw.cpu().numpy()[..., : s.C], ref) <= CONV_TOL, s

    net.train_step(lam)
    torch.cuda.synchronize()
    check([t["w"] for t in host])
    net.optimizer_step(0.0, 1e-4, 0.0, 0.0)     # w <- w - lr * dw: every weight moves, off the bf16 grid
    net.train_step(lam)
    torch.cuda.synchronize()
    new_w = [l.w_master.cpu().numpy()[..., : l.spec.C] for l in net.layers]
    assert not np.array_equal(new_w[1], host[1]["w"])
    check(new_w)


# ---------------------------------------------------------------------------------------------- #
# reconfiguration chain on whole networks
# ---------------------------------------------------------------------------------------------- #
def _oracle_chain(specs, edges, weights, thr):
    zo, zi = [], []
    for w in weights:
        on, inn = oracle.group_norms(w)
        # the device decides in fp32: round the fp64 norms to fp32 before the strict comparison
        zo.append(oracle.zero_groups(on.astype(np.float32), thr))
        zi.append(oracle.zero_groups(inn.astype(np.float32), thr))
    keep = [oracle.reconcile_edge([zo[i] for i in e.producers], [zi[i] for i in e.consumers]) for e in edges]
    idx = [oracle.compact_plan(k) for k in keep]
    return zo, zi, keep, idx


def _check_reconfig(specs, edges, weights, zero_sets, seed, thr, act_rows=0):
    from paper_1901_09290_amd import harness as hz
    model = hz.ReconfigModel(specs, edges, weights, seed=seed, with_activations=act_rows > 0)
    model.sweep(thr)
    torch.cuda.synchronize()
    zo, zi, keep, idx = _oracle_chain(specs, edges, weights, thr)
    cnt = model.new_counts
    for e, edge in enumerate(edges):
        assert np.array_equal(model.keep[e].cpu().numpy(), keep[e]), ("keep", e)
        assert int(cnt[e]) == idx[e].size, ("count", e)
        assert np.array_equal(model.idx[e].cpu().numpy()[: idx[e].size], idx[e]), ("idx", e)
        if zero_sets is not None:   # the planted pattern is what comes out
            assert np.array_equal(np.flatnonzero(keep[e] == 0), np.sort(zero_sets[e])), ("planted", e)
    rng = np.random.Generator(np.random.PCG64(seed))
    for i, s in enumerate(specs):
        assert np.array_equal(model.zo[i].cpu().numpy(), zo[i]) and np.array_equal(model.zi[i].cpu().numpy(), zi[i])
        ik = idx[s.out_edge] if s.out_edge is not None else None
        ic = idx[s.in_edge] if s.in_edge is not None else None
        Kp = s.K if ik is None else ik.size
        Cp = s.C if ic is None else ic.size
        op = hz.pitch8(Cp)
        for src, out in ((model.w[i], model.w_out[i]), (model.mom[i], model.mom_out[i])):
            host = src.cpu().numpy()[..., : s.C]
            got = out.reshape(-1)[: Kp * s.R * s.S * op].reshape(Kp, s.R, s.S, op).cpu().numpy()[..., :Cp]
            assert np.array_equal(got, oracle.compact_weights(host, ik, ic).astype(np.float32)), ("weights", i)
        if ik is not None:
            for v, o in zip(model.bn[i], model.bn_out[i]):
                assert np.array_equal(o.cpu().numpy()[:Kp], oracle.compact_vector(v.cpu().numpy(), ik)), ("vector", i)
        if act_rows and ic is not None:
            pixels = s.N * s.H * s.W
            rows = wl.sample_indices(pixels, act_rows, rng)
            rows = np.unique(np.concatenate([rows, [0, pixels - 1]]))
            rt = torch.from_numpy(rows).to(model.act[i].device)
            src = model.act[i].reshape(pixels, -1).view(torch.int16)[rt].cpu().numpy().view(np.uint16)[:, : s.C]
            out = model.act_out[i].reshape(-1)[: pixels * op].reshape(pixels, op).view(torch.int16)[rt]
            got = out.cpu().numpy().view(np.uint16)[:, :Cp]
            assert np.array_equal(got, oracle.compact_nhwc(src, ic)), ("activations", i)


def test_cfg2_resnet32_reconfiguration_chain():
    """ResNet-32 at batch 128: every residual stage is one edge with many producers and consumers."""
    specs, edges = wl.resnet32_layers(N=128)
    rng = np.random.Generator(np.random.PCG64(1))
    zero_sets = wl.zeroed_channel_sets(edges, 0.3, rng)
    weights = wl.network_weights(specs, edges, zero_sets, rng)
    _check_reconfig(specs, edges, weights, zero_sets, seed=1, thr=1e-6, act_rows=4096)


@pytest.mark.parametrize("seed", [10, 11, 12, 13, 14])
def test_cfg5_resnet50_reconfiguration_sweep(seed):
    """The benchmark's sweep: ResNet-50 at the pruned widths of cfg4, sparsity (seed-10)/10 of the channels
    of every edge zeroed; seed 13 (30 %) is the timed case and also checks the activation gathers at batch 64."""
    specs, edges = wl.resnet50_layers(N=64)
    keep = wl.pruned_keep_sets(edges, seed=3)
    pspecs, pedges = wl.with_widths(specs, edges, [k.size for k in keep])
    sparsity = (seed - 10) / 10.0
    rng = np.random.Generator(np.random.PCG64(seed))
    zero_sets = wl.zeroed_channel_sets(pedges, sparsity, rng)
    weights = wl.network_weights(pspecs, pedges, zero_sets, rng)
    _check_reconfig(pspecs, pedges, weights, zero_sets, seed=11, thr=1e-6, act_rows=2048 if seed == 13 else 0)


# ---------------------------------------------------------------------------------------------- #
# HIP graph: replays equal the eager launches
# ---------------------------------------------------------------------------------------------- #
def test_hip_graph_replays_equal_eager():
    """The benchmark replays captured launch sequences.  Capture a training step of a small network
    (stride-2, ragged and folded layers) plus the sweep's detection; replay it several times with eager
    work and synchronisation in between; every replay must reproduce the eager results bit for bit."""
    from paper_1901_09290_amd import harness as hz
    specs = [
        wl.ConvSpec("g0", 8, 32, 32, 3, 24, 3, 3, 1, 1, None, 0, first=True),
        wl.ConvSpec("g1", 8, 32, 32, 24, 40, 3, 3, 2, 1, 0, 1),
        wl.ConvSpec("g2", 8, 16, 16, 40, 72, 1, 1, 1, 0, 1, 2),
        wl.ConvSpec("g3", 8, 16, 16, 72, 72, 3, 3, 1, 1, 2, None),
        # a residual block with a shortcut convolution: the pair (b_a, b_proj) goes out as one batched forward call, the
        # shortcut's input gradient runs on a side stream, and b_b takes the kernel with the filter bank in LDS
        wl.ConvSpec("b_a", 8, 16, 16, 72, 32, 1, 1, 1, 0, 2, 3),
        wl.ConvSpec("b_b", 8, 16, 16, 32, 32, 3, 3, 1, 1, 3, 4),
        wl.ConvSpec("b_c", 8, 16, 16, 32, 96, 1, 1, 1, 0, 4, 5),
        wl.ConvSpec("b_proj", 8, 16, 16, 72, 96, 1, 1, 1, 0, 2, 5),
    ]
    edges = [wl.Edge("e0", 24, [0], [1]), wl.Edge("e1", 40, [1], [2]), wl.Edge("e2", 72, [2], [3, 4, 7]),
             wl.Edge("e3", 32, [4], [5]), wl.Edge("e4", 32, [5], [6]), wl.Edge("e5", 96, [6, 7], [])]
    net = hz.Network(hz.build_network(specs, seed=5))
    assert net.fork == {4: 7} and net.overlap_branches and net.batch_branches_fwd
    rng = np.random.Generator(np.random.PCG64(5))
    zero_sets = wl.zeroed_channel_sets(edges, 0.25, rng)
    model = hz.ReconfigModel(specs, edges, wl.network_weights(specs, edges, zero_sets, rng), seed=6)

    def snapshot():
        torch.cuda.synchronize()
        out = []
        for l in net.layers:
            out += [l.y.clone(), l.dw.clone(), l.out_norm.clone(), l.in_norm.clone()]
            if l.dx is not None:
                out.append(l.dx.clone())
        out += [k.clone() for k in model.keep] + [model.counts.clone()] + [i.clone() for i in model.idx]
        return out

    def scramble():
        for l in net.layers:
            l.y[..., : l.spec.K].fill_(1.0)      # logical elements only: the library never writes padding
            l.dw[..., : l.spec.C].fill_(-3.0)
            if l.dx is not None:
                l.dx[..., : l.spec.C].fill_(2.0)
        for k in model.keep:
            k.fill_(7)
        model.counts.fill_(-1)

    def eager():
        net.train_step(1e-3)
        model.detect(1e-6)

    eager()
    ref = snapshot()
    scramble()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            net.train_step(1e-3)
            model.detect(1e-6)
    torch.cuda.synchronize()
    for rep in range(4):
        scramble()
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, ref):
            assert torch.equal(a, b), rep
        # eager work of the same library between replays
        eager()
        torch.cuda.synchronize()
