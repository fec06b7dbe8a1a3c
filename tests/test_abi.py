"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-side argument validation answers with status codes before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

from paper_1901_09290_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B._SO):
        from paper_1901_09290_amd import build
        build.build()
    return B.lib()


def _declared():
    src = open(os.path.join(ROOT, "include", "prunetrain.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pt_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_weight_gradient_with_lasso_validates_before_launching(lib):
    d = B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1)
    n = C.c_size_t(0)
    assert lib.pt_conv_bwd_weight_lasso_workspace_bytes(C.byref(d), C.byref(n)) == 0
    assert n.value >= 16 * 9 * 16 * 4 and n.value >= B.conv_bwd_weight_workspace_bytes(d)   # at least one dw-sized slab
    assert lib.pt_conv_bwd_weight_lasso_workspace_bytes(C.byref(d), None) == -1
    fake = C.c_void_p(4096)
    args = lambda **kw: [kw.get(k, fake) for k in ("x", "dy", "w", "on", "inn")]
    call = lambda a, flags=3, ws=fake, nb=1 << 30: lib.pt_conv_bwd_weight_lasso(C.byref(d), a[0], a[1], a[2], a[3], a[4], 1e-3,
                                                                             flags, fake, ws, nb, None)
    for missing in ("x", "dy", "w", "on", "inn"):
        assert call(args(**{missing: None})) == -1
    assert call(args(), flags=4) == -4                     # unknown regulariser flag
    assert call(args(), ws=None) == -1                     # the slab is always needed
    assert call(args(), nb=16) == -3                       # workspace too small


def test_version(lib):
    assert lib.pt_version() >= 100


def test_workspace_queries_validate_descriptor(lib):
    d = B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1)
    assert B.conv_fwd_workspace_bytes(d) == 0
    assert B.conv_bwd_data_workspace_bytes(d) >= 16 * 9 * 16 * 2
    assert B.conv_bwd_weight_workspace_bytes(d) >= 0
    bad = B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1)
    bad.P = 15
    with pytest.raises(B.PruneTrainError) as e:
        B.conv_fwd_workspace_bytes(bad)
    assert e.value.status == -2
    bad = B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1, x_cpitch=8)
    with pytest.raises(B.PruneTrainError):
        B.conv_bwd_data_workspace_bytes(bad)
    bad = B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1)
    bad.struct_size = 12
    with pytest.raises(B.PruneTrainError):
        B.conv_bwd_weight_workspace_bytes(bad)
    assert B.conv_fwd_workspace_bytes(B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1, flags=B.CONV_PAD_ZERO)) == 0
    with pytest.raises(B.PruneTrainError) as e:
        B.conv_fwd_workspace_bytes(B.conv_desc(4, 16, 16, 16, 16, 3, 3, 1, 1, flags=2))     # unknown flag bit
    assert e.value.status == -4
    n = C.c_size_t(0)
    assert lib.pt_conv_fwd_workspace_bytes(None, C.byref(n)) == -1
    assert lib.pt_conv_fwd_workspace_bytes(C.byref(d), None) == -1
    huge = B.conv_desc(1 << 14, 1 << 10, 1 << 10, 8, 8, 1, 1, 1, 0)
    assert lib.pt_conv_fwd_workspace_bytes(C.byref(huge), C.byref(n)) == -4


def test_first_layer_weight_gradient_plan_and_workspace(lib):
    """An image-like first layer (at most 4 channels at a pitch of 8, at most 64 filters of at most 8 x 8, stride 1 or 2)
    takes its own weight-gradient kernel: one slab of [R][64][32] fp32 partial sums per workgroup, at most one
    workgroup per CU, always reduced.  Anything outside those limits keeps the general plan."""
    d = B.conv_desc(64, 224, 224, 3, 64, 7, 7, 2, 3, x_cpitch=8, y_cpitch=64, w_cpitch=8)
    info = B.conv_bwd_weight_plan(d, True)
    tiles = 64 * (112 // 2) * 2                      # tiles of 2 x 64 output pixels
    assert tiles == 7168 and info.splits == 256 and info.tiles == 1 and info.reduce_kind == B.WGRAD_REDUCE_DEEP
    assert B.conv_bwd_weight_workspace_bytes(d) >= 256 * 7 * 64 * 32 * 4
    assert B.conv_bwd_weight_lasso_workspace_bytes(d) >= 256 * 7 * 64 * 32 * 4
    small = B.conv_desc(2, 18, 18, 3, 16, 7, 7, 2, 3, x_cpitch=8, y_cpitch=16, w_cpitch=8)
    info = B.conv_bwd_weight_plan(small, True)
    assert info.splits == 2 * 5 * 1 and info.tiles == 1      # 9 x 9 outputs: five tile rows, one tile column
    # unaligned operands, a dense 3-channel pitch, or more than 64 filters: the general kernels
    assert B.conv_bwd_weight_plan(d, False).tiles > 1
    assert B.conv_bwd_weight_plan(B.conv_desc(64, 224, 224, 3, 64, 7, 7, 2, 3), True).tiles > 1
    wide = B.conv_desc(8, 64, 64, 3, 96, 3, 3, 1, 1, x_cpitch=8, y_cpitch=96, w_cpitch=8)
    assert B.conv_bwd_weight_plan(wide, True).tiles > 1


def test_batched_forward_validates_every_problem_before_launching(lib):
    d = B.conv_desc(2, 8, 8, 16, 16, 1, 1, 1, 0)
    bad = B.conv_desc(2, 8, 8, 16, 16, 1, 1, 1, 0)
    bad.P = 99
    two = (B.ConvDesc * 2)(d, bad)
    ptrs = (C.c_void_p * 2)(256, 256)       # never dereferenced: validation comes first
    assert lib.pt_conv_fwd_batched(two, ptrs, ptrs, ptrs, 2, None) == -2         # second descriptor inconsistent
    assert lib.pt_conv_fwd_batched(two, ptrs, ptrs, ptrs, 0, None) == -2         # no problems
    assert lib.pt_conv_fwd_batched(None, ptrs, ptrs, ptrs, 1, None) == -1
    assert lib.pt_conv_fwd_batched(two, None, ptrs, ptrs, 1, None) == -1
    holes = (C.c_void_p * 2)(256, None)
    good = (B.ConvDesc * 2)(d, d)
    assert lib.pt_conv_fwd_batched(good, ptrs, holes, ptrs, 2, None) == -1       # a NULL pointer in the second problem


def test_null_and_shape_errors_are_reported_before_launch(lib):
    d = B.conv_desc(1, 4, 4, 8, 8, 1, 1, 1, 0)
    assert lib.pt_conv_fwd(C.byref(d), None, None, None, None, 0, None) == -1
    assert lib.pt_conv_bwd_data(C.byref(d), None, None, None, None, 0, None) == -1
    assert lib.pt_conv_bwd_weight(C.byref(d), None, None, None, None, 0, None) == -1
    # workspace too small (non-null fake pointers are never dereferenced: validation fails first)
    fake = C.c_void_p(256)
    assert lib.pt_conv_bwd_data(C.byref(d), fake, fake, fake, fake, 16, None) == -3
    assert lib.pt_group_norms(None, 1, 1, 1, 1, None, None, None, None, 0, None) == -1
    assert lib.pt_group_norms(fake, 4, 1, 8, 4, fake, fake, None, fake, 1 << 20, None) == -2   # pitch < C
    assert lib.pt_group_norms(fake, 4, 1, 8, 8, fake, fake, None, fake, 0, None) == -3
    assert lib.pt_group_lasso_grad(fake, fake, fake, 0.1, 7, fake, 4, 1, 8, 8, None) == -4
    assert lib.pt_zero_groups(None, 0, 0.0, None, None) == 0
    assert lib.pt_zero_groups(None, 4, 0.0, None, None) == -1
    assert lib.pt_zero_groups(None, -1, 0.0, None, None) == -2
    assert lib.pt_reconcile_edge(None, 0, None, 0, 4, fake, None) == -2
    assert lib.pt_compact_plan(None, 4, None, None, None) == -1
    assert lib.pt_compact_weights(fake, 4, 1, 8, 8, None, 3, None, 8, fake, 8, None) == -2  # NULL idxK but Kp != K
    assert lib.pt_compact_vector(fake, 3, fake, 4, fake, None) == -4
    assert lib.pt_compact_vector(None, 4, None, 0, None, None) == 0
    assert lib.pt_compact_nhwc(fake, 10, 8, 8, fake, 9, fake, 16, None) == -2               # Cp > C
    assert lib.pt_compact_nhwc(None, 0, 8, 8, None, 4, None, 4, None) == 0


def test_batched_reconfiguration_calls_validate_on_the_host(lib):
    fake = 256
    assert lib.pt_zero_groups_batched(None, 0, 0.0, None) == 0
    assert lib.pt_zero_groups_batched(None, 3, 0.0, None) == -1
    assert lib.pt_zero_groups_batched(None, -1, 0.0, None) == -2
    jobs = (B.NormMask * 2)(B.NormMask(fake, fake, 0, 0), B.NormMask(None, fake, 4, 0))
    assert lib.pt_zero_groups_batched(jobs, 2, 0.0, None) == -1
    jobs = (B.NormMask * 1)(B.NormMask(fake, fake, -4, 0))
    assert lib.pt_zero_groups_batched(jobs, 1, 0.0, None) == -2
    assert lib.pt_reconcile_plan_batched(None, 2, None) == -1
    e = (B.EdgePlan * 1)(B.EdgePlan(None, None, 0, 0, 8, 0, fake, fake, fake))
    assert lib.pt_reconcile_plan_batched(e, 1, None) == -2          # an edge needs at least one member
    members = (C.c_void_p * 65)(*([fake] * 65))
    e = (B.EdgePlan * 1)(B.EdgePlan(C.cast(members, C.POINTER(C.c_void_p)), None, 65, 0, 8, 0, fake, fake, fake))
    assert lib.pt_reconcile_plan_batched(e, 1, None) == -4          # more than 64 members
    assert lib.pt_compact_vector_batched(None, 1, None) == -1
    v = (B.GatherVector * 1)(B.GatherVector(fake, fake, fake, 4, 3))
    assert lib.pt_compact_vector_batched(v, 1, None) == -4           # element size 3
    w = (B.GatherWeights * 1)(B.GatherWeights(fake, None, None, fake, 8, 1, 8, 8, 4, 8, 8, 0))
    assert lib.pt_compact_weights_batched(w, 1, None) == -2          # Kp != K without an index list
    assert lib.pt_compact_weights_batched(None, 0, None) == 0


def test_crsk_calls_validate_on_the_host(lib):
    fake = 256
    assert lib.pt_weights_to_crsk_batched(None, 0, None) == 0
    assert lib.pt_weights_to_crsk_batched(None, 2, None) == -1
    j = (B.LayerCrsk * 1)(B.LayerCrsk(fake, fake, 8, 9, 16, 8))
    assert lib.pt_weights_to_crsk_batched(j, 1, None) == -2          # pitch < C
    d = B.conv_desc(1, 4, 4, 8, 8, 1, 1, 1, 0)
    assert lib.pt_conv_bwd_data_crsk(C.byref(d), None, None, None, None) == -1
    assert lib.pt_conv_bwd_data_crsk(C.byref(d), fake, 8, fake, None) == -2   # wt not 16-byte aligned


def test_penalty_and_set_coeff_validate_on_the_host(lib):
    import oracle
    fake = 256
    assert lib.pt_group_lasso_penalty_batched(None, 0, None, None) == -1       # no result pointer
    assert lib.pt_group_lasso_penalty_batched(None, 2, fake, None) == -1
    j = (B.LayerPenalty * 1)(B.LayerPenalty(fake, fake, -1, 4, 3, 0))
    assert lib.pt_group_lasso_penalty_batched(j, 1, fake, None) == -2
    j = (B.LayerPenalty * 1)(B.LayerPenalty(fake, fake, 4, 4, 8, 0))
    assert lib.pt_group_lasso_penalty_batched(j, 1, fake, None) == -4          # unknown flag bit
    j = (B.LayerPenalty * 1)(B.LayerPenalty(None, fake, 4, 4, 3, 0))
    assert lib.pt_group_lasso_penalty_batched(j, 1, fake, None) == -1
    # SetCoeff is pure host arithmetic: identical to the oracle's, refuses what the oracle refuses
    for l1, l2, r in ((36.0, 12.0, 0.25), (2.3, 5311.7, 0.2), (0.0, 3.0, 0.5)):
        assert B.lasso_set_coeff(l1, l2, r) == oracle.set_coeff(l1, l2, r)
    for bad in ((1.0, 10.0, 0.0), (1.0, 10.0, 1.0), (1.0, 0.0, 0.2), (-1.0, 10.0, 0.2), (1.0, 10.0, float("nan"))):
        with pytest.raises(B.PruneTrainError) as e:
            B.lasso_set_coeff(*bad)
        assert e.value.status == -2
    assert lib.pt_lasso_set_coeff(1.0, 1.0, 0.5, None) == -1


def test_activation_gather_batched_validates_on_the_host(lib):
    fake = 256
    assert lib.pt_compact_nhwc_batched(None, 0, None) == 0
    assert lib.pt_compact_nhwc_batched(None, 2, None) == -1
    assert lib.pt_compact_nhwc_batched(None, -1, None) == -2
    j = (B.GatherNhwc * 2)(B.GatherNhwc(fake, fake, fake, 0, 8, 8, 4, 4), B.GatherNhwc(fake, fake, fake, 10, 8, 8, 9, 16))
    assert lib.pt_compact_nhwc_batched(j, 2, None) == -2             # Cp > C in the second job: nothing is launched
    j = (B.GatherNhwc * 1)(B.GatherNhwc(None, fake, fake, 10, 8, 8, 4, 4))
    assert lib.pt_compact_nhwc_batched(j, 1, None) == -1
    j = (B.GatherNhwc * 1)(B.GatherNhwc(None, None, None, 0, 8, 8, 4, 4))
    assert lib.pt_compact_nhwc_batched(j, 1, None) == 0              # an empty tensor needs no pointers


def test_gating_pieces_validate_on_the_host(lib):
    fake = 256
    assert lib.pt_scatter_nhwc(fake, 10, 5, 8, fake, 4, fake, 8, None) == -2      # Cp > C
    assert lib.pt_scatter_nhwc(fake, 10, 4, 8, fake, 9000, fake, 9000, None) == -4
    assert lib.pt_scatter_nhwc(None, 10, 4, 8, fake, 8, fake, 8, None) == -1
    assert lib.pt_scatter_nhwc(None, 0, 4, 8, None, 8, None, 8, None) == 0
    assert lib.pt_group_maxabs(fake, 4, 1, 8, 4, fake, fake, None) == -2            # pitch < C
    assert lib.pt_group_maxabs(fake, 4, 1, 4096, 4096, fake, fake, None) == -4
    assert lib.pt_group_maxabs(None, 4, 1, 8, 8, fake, fake, None) == -1
    assert lib.pt_apply_zero(None, 4, 1, 8, 8, fake, fake, None) == -1
    assert lib.pt_apply_zero(fake, 4, 1, 8, 4, fake, fake, None) == -2
    assert lib.pt_apply_zero(fake, 4, 1, 8, 8, None, None, None) == 0               # nothing flagged: nothing to do


def test_optimizer_step_validates_on_the_host(lib):
    fake = 256
    assert lib.pt_sgd_momentum_lasso_batched(None, 0, 0.1, 0.1, 0.9, 0.0, None) == 0
    assert lib.pt_sgd_momentum_lasso_batched(None, 1, 0.1, 0.1, 0.9, 0.0, None) == -1
    j = (B.LayerUpdate * 1)(B.LayerUpdate(fake, fake, None, fake, fake, 4, 1, 8, 8, 3, 0))
    assert lib.pt_sgd_momentum_lasso_batched(j, 1, 0.1, 0.1, 0.9, 0.0, None) == -1      # no momentum buffer
    j = (B.LayerUpdate * 1)(B.LayerUpdate(fake, fake, fake, fake, fake, 4, 1, 8, 4, 3, 0))
    assert lib.pt_sgd_momentum_lasso_batched(j, 1, 0.1, 0.1, 0.9, 0.0, None) == -2      # pitch < C
    j = (B.LayerUpdate * 1)(B.LayerUpdate(fake, fake, fake, fake, fake, 4, 1, 8, 8, 4, 0))
    assert lib.pt_sgd_momentum_lasso_batched(j, 1, 0.1, 0.1, 0.9, 0.0, None) == -4      # unknown flag bit


def test_feature_normalisation_validates_on_the_host(lib):
    import ctypes as C
    fake = 256
    n = C.c_size_t(0)
    assert lib.pt_bn_workspace_bytes(1000, 64, C.byref(n)) == 0 and n.value >= 2 * 64 * 4
    assert lib.pt_bn_workspace_bytes(1000, 64, None) == -1
    assert lib.pt_bn_workspace_bytes(0, 64, C.byref(n)) == -2
    assert lib.pt_bn_workspace_bytes(1000, 4096, C.byref(n)) == -4
    ok = (fake, 1000, 60, 64, fake, fake, 1e-5, fake, 64, fake, fake, fake, 1 << 30, None)

    def fwd(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return lib.pt_bn_fwd(*a)
    assert fwd(a0=None) == -1 and fwd(a4=None) == -1 and fwd(a11=None) == -1
    assert fwd(a3=56) == -2                  # pitch < C
    assert fwd(a3=68) == -4                  # rows not 16-byte
    assert fwd(a0=258) == -4                 # base not 16-byte aligned
    assert fwd(a6=-1.0) == -2
    assert fwd(a12=16) == -3
    okb = (fake, fake, 1000, 60, 64, 64, fake, fake, fake, fake, 64, fake, fake, fake, 1 << 30, None)

    def bwd(**kw):
        a = list(okb)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return lib.pt_bn_bwd(*a)
    assert bwd(a1=None) == -1 and bwd(a12=None) == -1
    assert bwd(a5=32) == -2 and bwd(a10=72 + 4) == -4 and bwd(a14=0) == -3
    assert bwd(a3=4096, a4=4096, a5=4096, a10=4096) == -4


def test_fused_statistics_calls_validate_on_the_host(lib):
    import ctypes as C
    fake = 256
    d = B.conv_desc(4, 16, 16, 16, 24, 3, 3, 1, 1)
    n, k = C.c_size_t(0), C.c_int32(0)
    assert lib.pt_conv_fwd_stats_workspace_bytes(C.byref(d), C.byref(n), C.byref(k)) == 0
    assert k.value == 8 and n.value >= 2 * 8 * 24 * 4
    assert lib.pt_conv_fwd_stats_workspace_bytes(C.byref(d), None, C.byref(k)) == -1
    assert lib.pt_conv_fwd_stats(C.byref(d), fake, fake, fake, None, 1 << 20, None) == -1
    assert lib.pt_conv_fwd_stats(C.byref(d), fake, fake, fake, fake, 16, None) == -3
    odd = B.conv_desc(4, 16, 16, 13, 24, 3, 3, 1, 1, x_cpitch=16, w_cpitch=16)        # C % 8 != 0, padding not vouched for
    assert lib.pt_conv_fwd_stats(C.byref(odd), fake, fake, fake, fake, 1 << 20, None) == -4
    dense = B.conv_desc(4, 16, 16, 13, 24, 3, 3, 1, 1)                                  # pitch 13: element-wise path
    assert lib.pt_conv_fwd_stats(C.byref(dense), fake, fake, fake, fake, 1 << 20, None) == -4
    ok = (fake, 1000, 60, 64, fake, 8, fake, fake, 1e-5, fake, 64, fake, fake, None)

    def f(**kw):
        a = list(ok)
        for key, v in kw.items():
            a[int(key[1:])] = v
        return lib.pt_bn_fwd_from_sums(*a)
    assert f(a4=None) == -1 and f(a0=None) == -1
    assert f(a5=0) == -2 and f(a3=56) == -2 and f(a3=68) == -4 and f(a2=4096, a3=4096, a10=4096) == -4
