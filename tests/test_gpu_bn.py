"""GPU parity: feature normalisation forward / backward through the C ABI against the fp64 oracle.

Tolerances: per-channel statistics and parameter gradients (fp32 partial sums combined in fp64) 1e-5 in the
metric of gpu_util.rel_err; the bf16 tensors y and dx must land on the bf16 value nearest the oracle's fp64
result for nearly every element (fp32 evaluation may cross a rounding boundary now and then), and never be
further than one bf16 step away: |g - r| <= 2^-7 |r| + 1e-6 rms.
"""
import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import binding as B
from paper_1901_09290_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

STAT_TOL = 1e-5
EPS = 1e-5


def _inputs(pixels, C, seed):
    """Activations like a convolution's output: per-channel scale and offset vary; channel 0 is constant
    (variance 0), channel 1 sits far from zero against its spread (cancellation case)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    scale = np.exp(rng.uniform(-2.0, 1.0, size=C))
    shift = rng.standard_normal(C) * scale
    x = rng.standard_normal((pixels, C)) * scale + shift
    x[:, 0] = 0.75
    if C > 1:
        x[:, 1] = 8.0 + 0.5 * rng.standard_normal(pixels)
    x = wl.to_bf16_grid(x.astype(np.float32))
    dy = wl.to_bf16_grid((rng.standard_normal((pixels, C)) * 0.1).astype(np.float32))
    gamma = (1.0 + 0.2 * rng.standard_normal(C)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(C)).astype(np.float32)
    return x, dy, gamma, beta


def _bf16_close(got, ref, C):
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, C)
    got = np.asarray(got, dtype=np.float64).reshape(-1, C)
    rms = float(np.sqrt(np.mean(ref * ref)))
    bound = 2.0 ** -7 * np.abs(ref) + 1e-6 * rms + 1e-30
    assert np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / bound))
    nearest = wl.to_bf16_grid(ref.astype(np.float32)).astype(np.float64)
    return float(np.mean(got == nearest))


def _run(pixels, C, xp, yp, dyp, dxp, seed):
    from gpu_util import DEV, dev_bf16, empty_bf16, host_bf16, rel_err, workspace
    x, dy, gamma, beta = _inputs(pixels, C, seed)
    xd, dyd = dev_bf16(x, xp), dev_bf16(dy, dyp)
    gd, bd = torch.from_numpy(gamma).to(DEV), torch.from_numpy(beta).to(DEV)
    y, dx = empty_bf16((pixels, yp), fill=0x7FC0), empty_bf16((pixels, dxp), fill=0x7FC0)
    mean, invstd, dgamma, dbeta = (torch.full((C,), float("nan"), device=DEV) for _ in range(4))
    ws = workspace(B.bn_workspace_bytes(pixels, C))
    ws.fill_(0xFF)
    B.bn_fwd(xd, pixels, C, xp, gd, bd, EPS, y, yp, mean, invstd, ws)
    B.bn_bwd(xd, dyd, pixels, C, xp, dyp, gd, mean, invstd, dx, dxp, dgamma, dbeta, ws)
    torch.cuda.synchronize()

    ry, rmean, rinv = oracle.bn_fwd(x.astype(np.float64), gamma, beta, EPS)
    rdx, rdg, rdb = oracle.bn_bwd(x.astype(np.float64), dy.astype(np.float64), gamma, rmean, rinv)
    assert rel_err(mean.cpu().numpy(), rmean) <= STAT_TOL
    assert rel_err(invstd.cpu().numpy(), rinv) <= STAT_TOL
    assert rel_err(dbeta.cpu().numpy(), rdb) <= STAT_TOL
    assert rel_err(dgamma.cpu().numpy(), rdg) <= STAT_TOL
    # the constant channel: variance exactly 0, so invstd = 1/sqrt(eps), y = beta, dx follows the formula
    assert abs(invstd[0].item() - 1.0 / np.sqrt(EPS)) <= 1e-4 / np.sqrt(EPS)
    hit_y = _bf16_close(host_bf16(y, C), ry, C)
    hit_dx = _bf16_close(host_bf16(dx, C), rdx, C)
    assert hit_y >= 0.98 and hit_dx >= 0.98, (hit_y, hit_dx)
    c8 = (C + 7) // 8 * 8
    for t, p in ((y, yp), (dx, dxp)):
        raw = t.view(torch.int16)
        assert bool((raw[:, C:c8] == 0).all())              # padding inside the last vector: written as zero
        assert bool((raw[:, c8:] == 0x7FC0).all())          # further padding: untouched
    return x, dy, gamma, beta, xd, dyd, gd, bd, ws


# (pixels, C, x pitch, y pitch, dy pitch, dx pitch)
CASES = [
    (37, 5, 8, 8, 8, 8),
    (1, 8, 8, 8, 8, 8),                       # one pixel: every variance is 0
    (2, 1, 8, 16, 8, 24),
    (1000, 64, 64, 64, 64, 64),
    (3137, 203, 208, 216, 208, 224),          # ragged channel count, unequal pitches
    (50000, 16, 24, 16, 16, 24),              # many pixel ranges, few channels
    (64 * 14 * 14, 1024, 1024, 1024, 1024, 1024),
    (200, 2048, 2048, 2048, 2048, 2048),      # the channel limit
    (7, 2041, 2048, 2048, 2048, 2048),
    (9001, 811, 816, 816, 816, 816),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[:2])))
def test_bn_forward_backward_match_oracle(case):
    _run(*case, seed=sum(case))


def test_bn_is_run_to_run_identical_and_full_size():
    """A ResNet-50 stage-1 activation (batch 64, 56x56, 64 channels) compared element by element, twice."""
    from gpu_util import DEV, empty_bf16
    pixels, C = 64 * 56 * 56, 64
    x, dy, gamma, beta, xd, dyd, gd, bd, ws = _run(pixels, C, C, C, C, C, seed=77)
    outs = []
    for _ in range(2):
        y, dx = empty_bf16((pixels, C)), empty_bf16((pixels, C))
        mean, invstd, dgamma, dbeta = (torch.empty((C,), device=DEV) for _ in range(4))
        B.bn_fwd(xd, pixels, C, C, gd, bd, EPS, y, C, mean, invstd, ws)
        B.bn_bwd(xd, dyd, pixels, C, C, C, gd, mean, invstd, dx, C, dgamma, dbeta, ws)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (y.view(torch.int16), dx.view(torch.int16), mean, invstd, dgamma, dbeta)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


FUSED = [
    # N  H   W   C    K   R st pad
    (2, 12, 12, 64, 64, 3, 1, 1),
    (3, 9, 11, 24, 40, 3, 1, 1),
    (2, 14, 14, 128, 96, 1, 1, 0),
    (2, 15, 15, 40, 136, 3, 2, 1),
    (2, 30, 30, 3, 28, 7, 2, 3),       # image-like input, zero padding vouched for
    (2, 13, 13, 45, 38, 3, 1, 1),      # ragged both ways
    (4, 28, 28, 128, 128, 3, 1, 1),    # several pixel tiles, two wave rows per tile
    (1, 1, 1, 8, 8, 1, 1, 0),
]


@pytest.mark.parametrize("case", FUSED, ids=lambda c: "x".join(map(str, c)))
def test_conv_with_statistics_epilogue_feeds_the_normalisation(case):
    """pt_conv_fwd_stats + pt_bn_fwd_from_sums against the oracle's convolution, rounded to bf16 as stored, followed
    by the oracle's normalisation; and against the unfused GPU path (same y bit for bit, statistics to 1e-5)."""
    from gpu_util import CONV_TOL, DEV, dev_bf16, empty_bf16, host_bf16, pitch8, rel_err, workspace
    N, H, W, C, K, R, st, pad = case
    spec = wl.ConvSpec("t", N, H, W, C, K, R, R, st, pad, None, None)
    t = wl.conv_tensors(spec, np.random.Generator(np.random.PCG64(900 + sum(case))), want=("x", "w"))
    xp, yp = pitch8(C), pitch8(K)
    d = B.desc_of(spec, xp, yp, xp, B.CONV_PAD_ZERO)
    xd, wd = dev_bf16(t["x"], xp, 0), dev_bf16(t["w"], xp, 0)
    pixels = N * spec.P * spec.Q
    rng = np.random.Generator(np.random.PCG64(7))
    gamma = (1.0 + 0.2 * rng.standard_normal(K)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(K)).astype(np.float32)
    gd, bd = torch.from_numpy(gamma).to(DEV), torch.from_numpy(beta).to(DEV)

    nbytes, n_partial = B.conv_fwd_stats_workspace(d)
    assert n_partial == (pixels + 127) // 128
    sums = workspace(nbytes)
    sums.fill_(0xFF)
    y = empty_bf16((N, spec.P, spec.Q, yp), fill=0)
    z = empty_bf16((pixels, yp), fill=0x7FC0)
    mean, invstd = (torch.full((K,), float("nan"), device=DEV) for _ in range(2))
    B.conv_fwd_stats(d, xd, wd, y, sums)
    B.bn_fwd_from_sums(y, pixels, K, yp, sums, n_partial, gd, bd, EPS, z, yp, mean, invstd)
    # unfused path on the same inputs
    y2 = empty_bf16((N, spec.P, spec.Q, yp), fill=0)
    z2 = empty_bf16((pixels, yp), fill=0x7FC0)
    mean2, invstd2 = (torch.full((K,), float("nan"), device=DEV) for _ in range(2))
    B.conv_fwd(d, xd, wd, y2)
    ws = workspace(B.bn_workspace_bytes(pixels, K))
    B.bn_fwd(y2, pixels, K, yp, gd, bd, EPS, z2, yp, mean2, invstd2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    assert rel_err(mean.cpu().numpy(), mean2.cpu().numpy()) <= 1e-5
    assert rel_err(invstd.cpu().numpy(), invstd2.cpu().numpy()) <= 1e-5

    ry = oracle.conv_fwd(oracle.shape_of(spec), t["x"], t["w"])
    assert rel_err(host_bf16(y, K), ry) <= CONV_TOL
    ry_stored = wl.to_bf16_grid(ry.astype(np.float32)).astype(np.float64).reshape(pixels, K)
    rz, rmean, rinv = oracle.bn_fwd(ry_stored, gamma, beta, EPS)
    # the two sides round a few outputs to neighbouring bf16 values: the statistics agree to that (derived: one bf16
    # step on a fraction of elements moves a mean by << 1e-3 of the channel's spread)
    assert rel_err(mean.cpu().numpy(), rmean) <= 1e-3
    assert rel_err(invstd.cpu().numpy(), rinv) <= 1e-3
    assert rel_err(host_bf16(z, K), rz) <= CONV_TOL
