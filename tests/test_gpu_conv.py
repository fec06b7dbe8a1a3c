"""GPU parity: the three convolutions through the C ABI against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import workloads as wl
from paper_1901_09290_amd.workloads import ConvSpec

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _spec(N, H, W, C, K, R, st, pad):
    return ConvSpec("t", N, H, W, C, K, R, R, st, pad, None, None)


def _check_full(spec, seed, xp=None, yp=None, wp=None, pad_zero=False):
    from gpu_util import CONV_TOL, rel_err, run_conv_all, strict_rel_err
    rng = np.random.Generator(np.random.PCG64(seed))
    t = wl.conv_tensors(spec, rng)
    y, dx, dw = run_conv_all(spec, t["x"], t["w"], t["dy"], xp, yp, wp, pad_zero)
    s = oracle.shape_of(spec)
    refs = (oracle.conv_fwd(s, t["x"], t["w"]), oracle.conv_bwd_data(s, t["dy"], t["w"]),
            oracle.conv_bwd_weight(s, t["x"], t["dy"]))
    errs = tuple(rel_err(g, r) for g, r in zip((y, dx, dw), refs))
    assert max(errs) <= CONV_TOL, (spec, errs)
    # the plain element-wise relative error away from cancellation zeros obeys the same bound (bf16 rounding of an
    # output is 2^-9 relative; fp32 accumulation adds far less on elements of this size)
    strict = tuple(strict_rel_err(g, r) for g, r in zip((y, dx, dw), refs))
    assert max(strict) <= CONV_TOL, (spec, strict)
    return errs + strict


def test_cfg1_single_layer():
    from gpu_util import CONV_TOL, rel_err, run_conv_all
    c = wl.cfg1(0)
    spec = c["spec"]
    y, dx, dw = run_conv_all(spec, c["x"], c["w"], c["dy"])
    s = oracle.shape_of(spec)
    ry, rdx, rdw = (oracle.conv_fwd(s, c["x"], c["w"]), oracle.conv_bwd_data(s, c["dy"], c["w"]),
                    oracle.conv_bwd_weight(s, c["x"], c["dy"]))
    assert rel_err(y, ry) <= CONV_TOL and rel_err(dx, rdx) <= CONV_TOL and rel_err(dw, rdw) <= CONV_TOL
    # zeroed groups give exact zeros: outputs of zero filters, input gradients of zero input channels
    assert np.all(y[..., c["zero_out"]] == 0.0)
    assert np.all(dx[..., c["zero_in"]] == 0.0)


SMALL = [
    # N  H   W   C    K   R st pad    several tiles + ragged tails in every GEMM dimension
    (2, 12, 12, 64, 64, 3, 1, 1),
    (3, 9, 11, 24, 40, 3, 1, 1),
    (2, 14, 14, 128, 96, 1, 1, 0),
    (2, 15, 15, 40, 136, 3, 2, 1),
    (2, 16, 16, 64, 128, 1, 2, 0),
    (1, 37, 37, 8, 16, 7, 2, 3),
    (5, 7, 7, 264, 72, 3, 1, 1),
    (1, 20, 20, 16, 200, 1, 1, 0),
    (1, 1, 1, 8, 8, 1, 1, 0),          # a single pixel
    (2, 5, 5, 8, 8, 5, 1, 0),          # filter as large as the image
    (1, 8, 8, 8, 8, 3, 3, 1),          # stride 3: parity classes with uneven tap counts
]


@pytest.mark.parametrize("case", SMALL)
def test_small_layers_full_tensor(case):
    _check_full(_spec(*case), seed=100 + sum(case))


RAGGED = [
    # logical C, K not multiples of 8; pitches padded to 8 (vector path with masked tails)
    ((2, 10, 10, 37, 51, 3, 1, 1), True),
    ((2, 12, 12, 203, 77, 1, 1, 0), True),
    ((1, 9, 9, 19, 131, 3, 2, 1), True),
    ((2, 18, 18, 3, 16, 7, 2, 3), True),   # image-like 3-channel input, pitch 8: filter rows folded into one run
    ((2, 30, 30, 3, 28, 7, 2, 3), True),
    ((3, 13, 13, 5, 24, 3, 1, 1), True),
    ((2, 11, 11, 12, 40, 5, 1, 2), True),  # pitch 16 with 12 real channels: a masked chunk inside every tap
    ((2, 9, 9, 32, 48, 2, 1, 0), True),    # folded run of exactly 64 elements
    ((2, 20, 20, 45, 38, 3, 1, 1), True),  # folded runs of 48 with 45 real channels: a tail in every 64-block
    ((2, 20, 20, 63, 40, 3, 1, 1), True),  # one 64-block per tap, tail in its last chunk
    ((2, 14, 14, 209, 45, 1, 1, 0), True),  # tail only in the last of four blocks
    # same shapes stored dense: pitches are odd, element-wise path
    ((2, 10, 10, 37, 51, 3, 1, 1), False),
    ((1, 9, 9, 19, 131, 3, 2, 1), False),
    ((2, 18, 18, 3, 16, 7, 2, 3), False),  # image-like 3-channel input
]


@pytest.mark.parametrize("case,padded", RAGGED)
def test_ragged_channel_counts(case, padded):
    from gpu_util import pitch8
    spec = _spec(*case)
    if padded:
        _check_full(spec, 200 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C))
    else:
        _check_full(spec, 300 + sum(case))


@pytest.mark.parametrize("case", [c for c, padded in RAGGED if padded] + [(2, 20, 20, 45, 38, 3, 1, 1),
                                                                          (2, 20, 20, 63, 40, 3, 1, 1),
                                                                          (2, 14, 14, 209, 45, 1, 1, 0)])
def test_ragged_channel_counts_with_zero_padding_vouched(case):
    """PT_CONV_PAD_ZERO: the inputs' padding channels are zero and the kernels skip clearing them."""
    from gpu_util import pitch8
    spec = _spec(*case)
    _check_full(spec, 400 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C), pad_zero=True)


MANY_TILES = [
    # launches with more tiles than the chip holds workgroups at once (650 - 770 pixel tiles, all whole), in both
    # pipeline depths of the direct kernel and with one, two, four and nine reduction steps per tile
    ((5, 128, 130, 64, 64, 1, 1, 0), False),    # one step per tile, three stages; input gradient alike
    ((5, 128, 130, 64, 128, 1, 1, 0), False),   # one step per tile, two stages; input gradient: two steps
    ((5, 128, 130, 128, 128, 1, 1, 0), False),  # two steps per tile, two stages, both directions
    ((7, 128, 100, 24, 64, 1, 1, 0), False),    # partial 64-channel block
    ((5, 128, 130, 64, 64, 3, 1, 1), False),    # nine steps per tile, image borders
    ((17, 128, 160, 64, 64, 2, 2, 0), False),   # strided: four input-gradient classes, scattered destination pixels
    ((6, 256, 256, 3, 64, 7, 2, 3), True),      # image-like input, filter rows folded, zero padding vouched for
    # 1 x 1 layers with several resident rounds of tiles: ragged channel counts on either side, an odd pixel count (the
    # last tile is partial and the last pixel has no partner in the paired stores)
    ((17, 55, 55, 40, 209, 1, 1, 0), True),     # forward: 402 x 2 tiles of 128 x 128, one partial reduction step
    ((24, 55, 55, 209, 33, 1, 1, 0), True),     # forward: 568 narrow tiles, four steps; input gradient: 568 x 2 tiles
    ((9, 128, 128, 72, 136, 1, 1, 0), False),   # channel counts multiples of 8 but not of 64, padding not vouched for
]


@pytest.mark.parametrize("case,pad_zero", MANY_TILES, ids=lambda c: "x".join(map(str, c)) if isinstance(c, tuple) else str(c))
def test_many_whole_tiles(case, pad_zero):
    from gpu_util import pitch8
    spec = _spec(*case)
    _check_full(spec, 600 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C), pad_zero=pad_zero)


FIRST_LAYER = [
    # image-like inputs (at most 4 channels at a pitch of 8, zero padding vouched for): the first-layer forward kernel
    (2, 33, 35, 1, 20, 3, 1, 1),      # one channel, 3 x 3 at stride 1 (one step per filter row)
    (3, 40, 70, 2, 70, 5, 1, 2),      # two channels, 5 x 5, two output-channel tiles with a ragged second one
    (2, 41, 150, 4, 64, 7, 1, 3),     # four channels, 7 x 7 at stride 1, rows of three tiles (the last partial)
    (2, 37, 37, 3, 40, 3, 2, 1),      # 3 x 3 at stride 2
    (2, 50, 50, 3, 100, 5, 2, 2),     # 5 x 5 at stride 2 (filter rows past the fifth multiply zeros)
    (2, 24, 24, 4, 24, 8, 2, 3),      # the largest filter the kernel takes
    (2, 10, 10, 4, 16, 1, 1, 0),      # a single tap
    (3, 21, 21, 3, 12, 2, 2, 0),      # 2 x 2 at stride 2, no padding
    (41, 200, 120, 3, 45, 7, 2, 3),   # 1025 tiles: runs of three tiles per workgroup, the last run of two
    (11, 200, 200, 3, 64, 7, 2, 3),   # 550 tiles: runs of two, alternating between the columns of a tile row
]


@pytest.mark.parametrize("case", FIRST_LAYER, ids=lambda c: "x".join(map(str, c)))
def test_image_like_first_layer(case):
    from gpu_util import pitch8
    spec = _spec(*case)
    _check_full(spec, 800 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C), pad_zero=True)


@pytest.mark.parametrize("case", [(8, 256, 256, 8, 16, 1, 1, 0), (2, 515, 511, 5, 24, 3, 1, 1), (3, 420, 420, 16, 64, 1, 1, 0)],
                         ids=lambda c: "x".join(map(str, c)))
def test_narrow_outputs_over_very_many_pixels(case):
    """More than half a million output pixels with at most 64 output channels: the forward launch takes 256-pixel tiles
    (whole and ragged pixel counts, plain / folded / partial-block reductions)."""
    from gpu_util import pitch8
    spec = _spec(*case)
    _check_full(spec, 700 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C), pad_zero=True)


EARLY_3X3 = [
    # 3 x 3, stride 1, padding 1, at most 64 channels on either side: the kernel that keeps the filter bank in LDS
    # (forward and input gradient); tiles are 4 rows x up to 56 columns
    ((2, 56, 56, 64, 64, 3, 1, 1), False),     # the shape it is for: one tile column of seven 8-pixel blocks
    ((3, 30, 70, 64, 64, 3, 1, 1), False),     # two tile columns (the second partial), a partial last tile row
    ((2, 13, 21, 40, 24, 3, 1, 1), False),     # three column blocks, 24 outputs: one accumulator block, 40 inputs: 2.5 steps
    ((2, 9, 5, 8, 8, 3, 1, 1), False),         # narrower than one block, a single 8-channel chunk
    ((2, 17, 33, 45, 38, 3, 1, 1), True),      # ragged counts, zero padding vouched for
    ((2, 20, 20, 26, 40, 3, 1, 1), True),
    ((2, 6, 60, 33, 56, 3, 1, 1), True),
    ((20, 56, 56, 32, 64, 3, 1, 1), False),    # 280 tiles: runs of two tiles per workgroup, the last run of one
    ((37, 28, 28, 16, 48, 3, 1, 1), False),    # 259 tiles of four blocks
    ((2, 20, 20, 48, 64, 3, 1, 1), False),     # input gradient: four 16-channel steps per tap and two accumulator blocks
]


@pytest.mark.parametrize("case,pad_zero", EARLY_3X3, ids=lambda c: "x".join(map(str, c)) if isinstance(c, tuple) else str(c))
def test_early_3x3_layers_with_resident_weights(case, pad_zero):
    from gpu_util import pitch8
    spec = _spec(*case)
    _check_full(spec, 950 + sum(case), pitch8(spec.C), pitch8(spec.K), pitch8(spec.C), pad_zero=pad_zero)


BATCHED_FWD = [
    # independent forward convolutions in one call: pairs that share a launch of the direct kernel (same tile shape and
    # variant: a block's first convolution and its strided shortcut), pairs that do not, and the other kernels mixed in
    [(4, 28, 28, 128, 64, 1, 1, 0), (4, 28, 28, 128, 256, 1, 2, 0)],          # 1x1 and strided 1x1 shortcut, same input shape
    [(6, 56, 56, 256, 128, 1, 1, 0), (6, 56, 56, 256, 512, 1, 2, 0)],         # both 128 x 128 tiles: one launch, two problems
    [(6, 56, 56, 209, 87, 1, 1, 0), (6, 56, 56, 209, 371, 1, 2, 0)],          # ragged widths
    [(2, 14, 14, 64, 64, 3, 1, 1), (2, 14, 14, 64, 256, 1, 1, 0), (2, 14, 14, 64, 64, 1, 1, 0)],   # three problems, mixed shapes
    [(2, 18, 18, 3, 16, 7, 2, 3), (2, 12, 12, 24, 40, 3, 1, 1)],               # an image-like first layer beside a 3 x 3 layer
    [(2, 9, 9, 16, 24, 1, 1, 0)] * 5,                                          # more problems than one launch holds
]


@pytest.mark.parametrize("cases", BATCHED_FWD, ids=lambda cs: "+".join("x".join(map(str, c)) for c in cs)[:60])
def test_batched_forward_against_oracle_and_single_calls(cases):
    """pt_conv_fwd_batched: every problem's output against the oracle and bit for bit against pt_conv_fwd alone."""
    from gpu_util import CONV_TOL, DEV, dev_bf16, host_bf16, pitch8, rel_err
    from paper_1901_09290_amd import binding as B
    specs = [_spec(*c) for c in cases]
    rng = np.random.Generator(np.random.PCG64(900 + sum(map(sum, cases))))
    descs, xs, ws, ys, singles, refs = [], [], [], [], [], []
    for spec in specs:
        t = wl.conv_tensors(spec, rng, want=("x", "w"))
        xp, yp, wp = pitch8(spec.C), pitch8(spec.K), pitch8(spec.C)
        d = B.desc_of(spec, xp, yp, wp, B.CONV_PAD_ZERO)
        x, w = dev_bf16(t["x"], xp, pad=0), dev_bf16(t["w"], wp, pad=0)   # zero padding, as vouched for
        y = torch.full((spec.N, spec.P, spec.Q, yp), -1, dtype=torch.int16, device=DEV)
        y1 = torch.full_like(y, -1)
        B.conv_fwd(d, x, w, y1)
        descs.append(d); xs.append(x); ws.append(w); ys.append(y); singles.append(y1)
        refs.append(oracle.conv_fwd(oracle.shape_of(spec), t["x"], t["w"]))
    B.conv_fwd_batched(B.conv_fwd_jobs(descs, xs, ws, ys))
    torch.cuda.synchronize()
    for spec, y, y1, ref in zip(specs, ys, singles, refs):
        assert torch.equal(y, y1), spec
        assert rel_err(host_bf16(y, spec.K), ref) <= CONV_TOL, spec


FUSED_LASSO = [
    # N  H   W   C    K   R st pad   flags  path    reductions split over many workgroups, and single-slab ones
    ((2, 12, 12, 64, 64, 3, 1, 1), 3, None),
    ((3, 9, 11, 24, 40, 3, 1, 1), 3, None),
    ((2, 14, 14, 128, 96, 1, 1, 0), 1, None),
    ((2, 15, 15, 40, 136, 3, 2, 1), 2, None),
    ((2, 18, 18, 3, 16, 7, 2, 3), 1, None),          # a first layer: input groups exempt
    ((2, 10, 10, 37, 51, 3, 1, 1), 3, None),         # ragged counts
    ((1, 7, 7, 520, 520, 3, 1, 1), 3, "none"),       # more tiles than the split target: one slab, no split
    ((5, 128, 130, 64, 64, 1, 1, 0), 3, "deep"),     # very many pixels: many slices over few outputs
    # few slices over many outputs (the late layers of a deep network): the wide reduction adds the regulariser
    ((8, 14, 14, 256, 256, 3, 1, 1), 3, "wide"),
    ((8, 14, 14, 203, 171, 3, 1, 1), 3, "wide"),     # the same with ragged counts
    ((8, 14, 14, 203, 171, 3, 1, 1), 1, "wide"),
    ((8, 14, 14, 203, 171, 3, 1, 1), 2, "wide"),
    ((16, 14, 14, 520, 264, 1, 1, 0), 3, "wide"),
]


@pytest.mark.parametrize("case,flags,path", FUSED_LASSO,
                         ids=lambda c: "x".join(map(str, c)) if isinstance(c, tuple) else str(c))
@pytest.mark.parametrize("padded", [True, False])
def test_weight_gradient_with_regulariser_folded_in(case, flags, path, padded):
    """pt_conv_bwd_weight_lasso against the oracle's weight gradient plus the oracle's lasso gradient (convolution
    tolerance on the sum, 1e-5 on the added term itself), and against the two separate GPU calls.  Where a case is
    meant for one of the reduction passes, the library's own plan must say that it takes it."""
    from gpu_util import CONV_TOL, DEV, F32_TOL, dev_bf16, dev_f32, pitch8, rel_err, workspace
    from paper_1901_09290_amd import binding as B
    spec = _spec(*case)
    if path is not None and padded:
        info = B.conv_bwd_weight_plan(B.desc_of(spec, pitch8(spec.C), pitch8(spec.K), pitch8(spec.C)), True)
        kinds = {"none": B.WGRAD_REDUCE_NONE, "deep": B.WGRAD_REDUCE_DEEP, "wide": B.WGRAD_REDUCE_WIDE}
        assert info.reduce_kind == kinds[path], (case, info.splits, info.tiles, info.reduce_kind)
        assert (info.splits == 1) == (path == "none")
    rng = np.random.Generator(np.random.PCG64(800 + sum(case) + flags))
    t = wl.conv_tensors(spec, rng, want=("x", "dy"))
    w = (rng.standard_normal((spec.K, spec.R, spec.S, spec.C)) * 0.05).astype(np.float32)
    w[0] = 0.0                    # a zero output group and a zero input group: their terms are exactly 0
    w[..., spec.C - 1] = 0.0
    lam = 0.5                     # large, so that the added term is visible beside the data gradient
    xp, yp, wp = (pitch8(spec.C), pitch8(spec.K), pitch8(spec.C)) if padded else (spec.C, spec.K, spec.C)
    d = B.desc_of(spec, xp, yp, wp)
    xd, dyd, wd = dev_bf16(t["x"], xp), dev_bf16(t["dy"], yp), dev_f32(w, wp)
    ron, rin = oracle.group_norms(w)
    on = torch.from_numpy(ron.astype(np.float32)).to(DEV)
    inn = torch.from_numpy(rin.astype(np.float32)).to(DEV)
    RS = spec.R * spec.S
    ws = workspace(max(B.conv_bwd_weight_lasso_workspace_bytes(d), B.conv_bwd_weight_workspace_bytes(d)))
    dw_f = torch.full((spec.K, spec.R, spec.S, wp), float("nan"), dtype=torch.float32, device=DEV)
    dw_s = torch.full((spec.K, spec.R, spec.S, wp), float("nan"), dtype=torch.float32, device=DEV)
    B.conv_bwd_weight_lasso(d, xd, dyd, wd, on, inn, lam, flags, dw_f, ws)
    B.conv_bwd_weight(d, xd, dyd, dw_s, ws)
    torch.cuda.synchronize()
    plain = dw_s.cpu().numpy()[..., : spec.C].copy()
    B.group_lasso_grad(wd, on, inn, lam, flags, dw_s, spec.K, RS, spec.C, wp)
    torch.cuda.synchronize()
    fused, separate = dw_f.cpu().numpy()[..., : spec.C], dw_s.cpu().numpy()[..., : spec.C]
    if wp != spec.C:
        assert bool(torch.isnan(dw_f[..., spec.C:]).all())              # padding untouched
    rdw = oracle.conv_bwd_weight(oracle.shape_of(spec), t["x"], t["dy"])
    ref = oracle.group_lasso_grad(w, on.cpu().numpy(), inn.cpu().numpy(), lam, flags, rdw)
    assert rel_err(fused, ref) <= CONV_TOL
    # the added term alone: what the fused call wrote minus the plain weight gradient of the same kernels
    term_ref = oracle.group_lasso_grad(w, on.cpu().numpy(), inn.cpu().numpy(), lam, flags, np.zeros_like(rdw))
    # (one fp32 rounding of the sum, a few ulps of the larger operand, plus 1e-5 of the term)
    big = np.maximum(np.abs(plain), np.abs(fused)).astype(np.float32)
    slack = 4 * np.spacing(big).astype(np.float64) + 1e-5 * (np.abs(term_ref) + np.sqrt(np.mean(term_ref ** 2)))
    assert np.all(np.abs(fused.astype(np.float64) - plain - term_ref) <= slack)
    assert rel_err(fused, separate) <= F32_TOL
    if flags == 1:
        assert np.array_equal(fused[0], plain[0])                       # zero output group: nothing added


def test_results_are_run_to_run_identical():
    from gpu_util import run_conv_all
    spec = _spec(4, 14, 14, 72, 104, 3, 1, 1)
    t = wl.conv_tensors(spec, np.random.Generator(np.random.PCG64(7)))
    a = run_conv_all(spec, t["x"], t["w"], t["dy"])
    b = run_conv_all(spec, t["x"], t["w"], t["dy"])
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_cfg2_resnet32_distinct_layers_full_tensor():
    """Every distinct layer shape of the ResNet-32-shaped stack at batch 128, whole tensors."""
    layers, _ = wl.resnet32_layers(N=128)
    rng_seed = 1
    for i, (spec, _) in enumerate(wl.distinct_shapes(layers)):
        errs = _check_full(spec, rng_seed * 1000 + i)
        print(spec.name, spec.shape_key(), "metric", ["%.2e" % e for e in errs[:3]], "element-wise", ["%.2e" % e for e in errs[3:]],
              flush=True)


@pytest.mark.parametrize("case", [(2, 15, 15, 40, 136, 3, 2, 1), (2, 10, 10, 37, 51, 3, 1, 1), (2, 16, 16, 64, 128, 1, 2, 0)])
def test_bwd_data_from_pretransposed_weights(case):
    """pt_weights_to_crsk_batched + pt_conv_bwd_data_crsk: the transposed copy is an exact permutation
    (k padding zero) and the input gradient is bit-identical to pt_conv_bwd_data's."""
    import torch
    from gpu_util import DEV, dev_bf16, empty_bf16, pitch8, workspace
    from paper_1901_09290_amd import binding as B
    spec = _spec(*case)
    t = wl.conv_tensors(spec, np.random.Generator(np.random.PCG64(900 + sum(case))))
    xp, yp, wp = pitch8(spec.C), pitch8(spec.K), pitch8(spec.C)
    d = B.desc_of(spec, xp, yp, wp)
    wd, dyd = dev_bf16(t["w"], wp), dev_bf16(t["dy"], yp)
    RS = spec.R * spec.S
    wt = torch.full((spec.C, RS, yp), float("nan"), dtype=torch.bfloat16, device=DEV)
    other = torch.full((7, 1, 8), float("nan"), dtype=torch.bfloat16, device=DEV)   # a second job in the same launch
    w2 = dev_bf16(np.arange(5 * 7, dtype=np.float32).reshape(5, 1, 7), 8)
    B.weights_to_crsk_batched([B.layer_crsk(wd, wt, spec.K, RS, spec.C, wp), B.layer_crsk(w2, other, 5, 1, 7, 8)])
    dx_a = empty_bf16((spec.N, spec.H, spec.W, xp), fill=0x7FC0)
    dx_b = empty_bf16((spec.N, spec.H, spec.W, xp), fill=0x7FC0)
    B.conv_bwd_data_crsk(d, dyd, wt, dx_a)
    B.conv_bwd_data(d, dyd, wd, dx_b, workspace(B.conv_bwd_data_workspace_bytes(d)))
    torch.cuda.synchronize()
    want = np.zeros((spec.C, RS, yp), dtype=np.float32)
    want[..., : spec.K] = t["w"].reshape(spec.K, RS, spec.C).transpose(2, 1, 0)
    assert np.array_equal(wt.float().cpu().numpy(), want)
    o = other.float().cpu().numpy()
    assert np.array_equal(o[:, 0, :5], np.arange(35, dtype=np.float32).reshape(5, 7).T) and not o[:, 0, 5:].any()
    assert torch.equal(dx_a.view(torch.int16), dx_b.view(torch.int16))


def _random_specs(n, seed):
    """Seeded random small layers: arbitrary (pruned-looking) channel counts, filter sizes 1/3/5/7, strides 1-3."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    while len(out) < n:
        R = int(rng.choice([1, 1, 3, 3, 5, 7]))
        stride = int(rng.choice([1, 1, 2, 3]))
        pad = int(rng.integers(0, R // 2 + 1))
        H, W = int(rng.integers(max(R, 4), 24)), int(rng.integers(max(R, 4), 24))
        C = int(rng.choice([rng.integers(1, 16), rng.integers(16, 80), rng.integers(80, 300)]))
        K = int(rng.choice([rng.integers(1, 16), rng.integers(16, 80), rng.integers(80, 300)]))
        N = int(rng.integers(1, 5))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        out.append((N, H, W, C, K, R, stride, pad))
    return out


@pytest.mark.parametrize("case", _random_specs(36, 20260101), ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("pad_zero", [False, True])
def test_random_ragged_layers(case, pad_zero):
    """Arbitrary widths on 8-padded pitches, padding NaN (kernels clear the tails) or vouched zero."""
    from gpu_util import pitch8
    N, H, W, C, K, R, stride, pad = case
    spec = _spec(N, H, W, C, K, R, stride, pad)
    _check_full(spec, 500 + sum(case), pitch8(C), pitch8(K), pitch8(C), pad_zero=pad_zero)
