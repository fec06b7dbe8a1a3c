"""The entry point that allocates nothing, pt_group_norms_static, against pt_group_norms (same kernels, the scratch
held by the library instead of a caller's workspace): two calls in a row, the second on a smaller layer, so that
whatever the first call left in the shared scratch must not leak into the second; then the oracle."""
import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import binding as B
from paper_1901_09290_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _both(w, pitch):
    from gpu_util import DEV, dev_f32, workspace
    K, C = w.shape[0], w.shape[-1]
    RS = w.size // (K * C)
    wd = dev_f32(w, pitch)
    out = {}
    for tag in ("static", "ws"):
        on = torch.full((K,), float("nan"), device=DEV)
        inn = torch.full((C,), float("nan"), device=DEV)
        sh = torch.empty((K, RS, pitch), dtype=torch.bfloat16, device=DEV)
        sh.view(torch.int16).fill_(0x7FC0)
        out[tag] = (on, inn, sh)
    ws = workspace(B.group_norms_workspace_bytes(K, RS, C))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.group_norms_static(wd, K, RS, C, pitch, *out["static"])
    assert torch.cuda.memory_allocated() == before
    B.group_norms(wd, K, RS, C, pitch, *out["ws"], ws)
    torch.cuda.synchronize()
    return out


def test_static_scratch_entry_point_matches_the_workspace_one():
    from gpu_util import F32_TOL, pitch8, rel_err
    rng = np.random.Generator(np.random.PCG64(4242))
    # large first (many chunks, all of the scratch layout in use), then smaller ones that reuse the same scratch
    for shape, padded in (((512, 3, 3, 512), True), ((203, 1, 1, 811), True), ((37, 3, 3, 51), True), ((64, 3, 3, 37), False),
                          ((512, 3, 3, 512), True)):
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.05)
        w[1] = 0.0
        w[..., 2] = 0.0
        pitch = pitch8(shape[-1]) if padded else shape[-1]
        out = _both(w, pitch)
        for a, b in zip(out["static"], out["ws"]):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a, b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
        ron, rin = oracle.group_norms(w)
        on, inn, sh = out["static"]
        assert rel_err(on.cpu().numpy(), ron) <= F32_TOL and rel_err(inn.cpu().numpy(), rin) <= F32_TOL
        assert on[1].item() == 0.0 and inn[2].item() == 0.0
        got = sh.view(torch.int16).cpu().numpy().view(np.uint16).reshape(shape[0], -1, pitch)[..., : shape[-1]]
        assert np.array_equal(got, wl.bf16_bits(wl.to_bf16_grid(w)).reshape(shape[0], -1, shape[-1]))


def test_static_scratch_entry_point_rejects_layers_beyond_its_scratch():
    from gpu_util import DEV
    K, RS, C = 4096, 9, 2048            # 75 M parameters: far beyond the 4 MiB of held scratch
    dummy = torch.zeros(16, device=DEV)
    with pytest.raises(B.PruneTrainError) as e:
        B.group_norms_static(dummy, K, RS, C, C, dummy, dummy, None)
    assert e.value.status == -3          # PT_ERR_WORKSPACE
