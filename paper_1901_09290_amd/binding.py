"""Thin ctypes binding of libprunetrain.so: same names as include/prunetrain.h without the pt_ prefix.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used for device memory
and streams, nothing else); every step of the path runs inside the HIP library.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libprunetrain.so")
_lib = None

PT_OK = 0
STATUS = {0: "PT_OK", -1: "PT_ERR_NULL", -2: "PT_ERR_SHAPE", -3: "PT_ERR_WORKSPACE", -4: "PT_ERR_UNSUPPORTED",
          -5: "PT_ERR_LAUNCH", -6: "PT_ERR_EMPTY"}
LASSO_OUT, LASSO_IN = 1, 2
EDGE_FED_OUTSIDE, EDGE_READ_OUTSIDE = 1, 2
CONV_PAD_ZERO = 1  # pt_conv_desc.flags: padding channels of the input tensors are zero

EXPORTS = [
    "pt_version", "pt_last_hip_error",
    "pt_conv_fwd_workspace_bytes", "pt_conv_bwd_data_workspace_bytes", "pt_conv_bwd_weight_workspace_bytes",
    "pt_conv_fwd", "pt_conv_fwd_batched", "pt_conv_bwd_data", "pt_conv_bwd_weight",
    "pt_group_norms_workspace_bytes", "pt_group_norms", "pt_group_lasso_grad",
    "pt_group_norms_batched_workspace_bytes", "pt_group_norms_batched", "pt_group_lasso_grad_batched",
    "pt_group_norms_detect_batched_workspace_bytes", "pt_group_norms_detect_batched", "pt_conv_bwd_weight_plan",
    "pt_group_norms_static",
    "pt_zero_groups", "pt_reconcile_edge", "pt_compact_plan",
    "pt_compact_weights", "pt_compact_vector", "pt_compact_nhwc",
    "pt_weights_to_crsk_batched", "pt_conv_bwd_data_crsk",
    "pt_group_lasso_penalty_batched", "pt_lasso_set_coeff", "pt_compact_nhwc_batched",
    "pt_scatter_nhwc", "pt_group_maxabs", "pt_apply_zero", "pt_sgd_momentum_lasso_batched",
    "pt_zero_groups_batched", "pt_reconcile_plan_batched", "pt_compact_vector_batched", "pt_compact_weights_batched",
    "pt_bn_workspace_bytes", "pt_bn_fwd", "pt_bn_bwd", "pt_plan_layer_removal",
    "pt_conv_fwd_stats_workspace_bytes", "pt_conv_fwd_stats", "pt_bn_fwd_from_sums",
    "pt_conv_bwd_weight_lasso_workspace_bytes", "pt_conv_bwd_weight_lasso",
]


class PruneTrainError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        hip = lib().pt_last_hip_error() if status == -5 else 0
        super().__init__(f"{call}: {STATUS.get(status, status)}" + (f" (hip error {hip})" if hip else ""))


class ConvDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_int32) for n in (
        "N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "P", "Q",
        "x_cpitch", "y_cpitch", "w_cpitch")] + [("flags", C.c_uint32)]


class LayerWeights(C.Structure):
    _fields_ = [("w", C.c_void_p), ("out_norm", C.c_void_p), ("in_norm", C.c_void_p), ("w_shadow", C.c_void_p),
                ("K", C.c_int32), ("RS", C.c_int32), ("C", C.c_int32), ("w_cpitch", C.c_int32)]


class LayerDetect(C.Structure):
    _fields_ = [("w", C.c_void_p), ("out_norm", C.c_void_p), ("in_norm", C.c_void_p), ("zero_out", C.c_void_p),
                ("zero_in", C.c_void_p), ("K", C.c_int32), ("RS", C.c_int32), ("C", C.c_int32), ("w_cpitch", C.c_int32)]


class WgradPlanInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("splits", "tiles", "reduce_kind", "tile_m", "tile_n")]


WGRAD_REDUCE_NONE, WGRAD_REDUCE_DEEP, WGRAD_REDUCE_WIDE = 0, 1, 2


class LayerLasso(C.Structure):
    _fields_ = [("w", C.c_void_p), ("out_norm", C.c_void_p), ("in_norm", C.c_void_p), ("dw", C.c_void_p),
                ("K", C.c_int32), ("RS", C.c_int32), ("C", C.c_int32), ("w_cpitch", C.c_int32),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class LayerCrsk(C.Structure):
    _fields_ = [("w", C.c_void_p), ("wt", C.c_void_p), ("K", C.c_int32), ("RS", C.c_int32), ("C", C.c_int32),
                ("w_cpitch", C.c_int32)]


class LayerPenalty(C.Structure):
    _fields_ = [("out_norm", C.c_void_p), ("in_norm", C.c_void_p), ("K", C.c_int32), ("C", C.c_int32),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class GatherNhwc(C.Structure):
    _fields_ = [("x", C.c_void_p), ("idx", C.c_void_p), ("out", C.c_void_p), ("pixels", C.c_int64),
                ("C", C.c_int32), ("x_cpitch", C.c_int32), ("Cp", C.c_int32), ("out_cpitch", C.c_int32)]


class LayerUpdate(C.Structure):
    _fields_ = [("w", C.c_void_p), ("dw", C.c_void_p), ("mom", C.c_void_p), ("out_norm", C.c_void_p),
                ("in_norm", C.c_void_p), ("K", C.c_int32), ("RS", C.c_int32), ("C", C.c_int32), ("w_cpitch", C.c_int32),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class NormMask(C.Structure):
    _fields_ = [("norms", C.c_void_p), ("zero", C.c_void_p), ("n", C.c_int32), ("reserved", C.c_int32)]


class EdgePlan(C.Structure):
    _fields_ = [("producer_zero", C.POINTER(C.c_void_p)), ("consumer_zero", C.POINTER(C.c_void_p)),
                ("n_prod", C.c_int32), ("n_cons", C.c_int32), ("n", C.c_int32), ("reserved", C.c_int32),
                ("keep", C.c_void_p), ("idx", C.c_void_p), ("n_keep_dev", C.c_void_p)]


class RemovalEdge(C.Structure):
    _fields_ = [("producers", C.POINTER(C.c_int32)), ("consumers", C.POINTER(C.c_int32)), ("n_prod", C.c_int32),
                ("n_cons", C.c_int32), ("n_keep", C.c_int32), ("external", C.c_int32)]


class GatherVector(C.Structure):
    _fields_ = [("v", C.c_void_p), ("idx", C.c_void_p), ("out", C.c_void_p), ("n_keep", C.c_int32),
                ("elem_bytes", C.c_int32)]


class GatherWeights(C.Structure):
    _fields_ = [("w", C.c_void_p), ("idxK", C.c_void_p), ("idxC", C.c_void_p), ("w_out", C.c_void_p)] + [
        (n, C.c_int32) for n in ("K", "RS", "C", "w_cpitch", "Kp", "Cp", "out_cpitch", "reserved")]


def lib() -> C.CDLL:
    """The loaded HIP library; loading failure is fatal (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise ImportError(f"{_SO} is not built: run `python -m paper_1901_09290_amd.build` "
                              "(or __graft_entry__.build()) first; there is no CPU fallback")
        _lib = C.CDLL(_SO)
        vp, i32, i64, u32, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_float, C.c_size_t
        dp = C.POINTER(ConvDesc)
        sig = {
            "pt_version": [], "pt_last_hip_error": [],
            "pt_conv_fwd_workspace_bytes": [dp, C.POINTER(sz)],
            "pt_conv_bwd_data_workspace_bytes": [dp, C.POINTER(sz)],
            "pt_conv_bwd_weight_workspace_bytes": [dp, C.POINTER(sz)],
            "pt_conv_fwd": [dp, vp, vp, vp, vp, sz, vp],
            "pt_conv_fwd_batched": [dp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i32, vp],
            "pt_conv_bwd_data": [dp, vp, vp, vp, vp, sz, vp],
            "pt_conv_bwd_weight": [dp, vp, vp, vp, vp, sz, vp],
            "pt_conv_bwd_weight_lasso_workspace_bytes": [dp, C.POINTER(sz)],
            "pt_conv_bwd_weight_lasso": [dp, vp, vp, vp, vp, vp, f32, u32, vp, vp, sz, vp],
            "pt_group_norms_workspace_bytes": [i32, i32, i32, C.POINTER(sz)],
            "pt_group_norms": [vp, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp],
            "pt_group_lasso_grad": [vp, vp, vp, f32, u32, vp, i32, i32, i32, i32, vp],
            "pt_group_norms_static": [vp, i32, i32, i32, i32, vp, vp, vp, vp],
            "pt_group_norms_batched_workspace_bytes": [C.POINTER(LayerWeights), i32, C.POINTER(sz)],
            "pt_group_norms_batched": [C.POINTER(LayerWeights), i32, vp, sz, vp],
            "pt_group_lasso_grad_batched": [C.POINTER(LayerLasso), i32, f32, vp],
            "pt_group_norms_detect_batched_workspace_bytes": [C.POINTER(LayerDetect), i32, C.POINTER(sz)],
            "pt_group_norms_detect_batched": [C.POINTER(LayerDetect), i32, f32, vp, sz, vp],
            "pt_conv_bwd_weight_plan": [dp, i32, C.POINTER(WgradPlanInfo)],
            "pt_zero_groups": [vp, i32, f32, vp, vp],
            "pt_reconcile_edge": [C.POINTER(vp), i32, C.POINTER(vp), i32, i32, vp, vp],
            "pt_compact_plan": [vp, i32, vp, vp, vp],
            "pt_compact_weights": [vp, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, vp],
            "pt_compact_vector": [vp, i32, vp, i32, vp, vp],
            "pt_compact_nhwc": [vp, i64, i32, i32, vp, i32, vp, i32, vp],
            "pt_weights_to_crsk_batched": [C.POINTER(LayerCrsk), i32, vp],
            "pt_conv_bwd_data_crsk": [dp, vp, vp, vp, vp],
            "pt_group_lasso_penalty_batched": [C.POINTER(LayerPenalty), i32, vp, vp],
            "pt_lasso_set_coeff": [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)],
            "pt_compact_nhwc_batched": [C.POINTER(GatherNhwc), i32, vp],
            "pt_sgd_momentum_lasso_batched": [C.POINTER(LayerUpdate), i32, f32, f32, f32, f32, vp],
            "pt_scatter_nhwc": [vp, i64, i32, i32, vp, i32, vp, i32, vp],
            "pt_group_maxabs": [vp, i32, i32, i32, i32, vp, vp, vp],
            "pt_apply_zero": [vp, i32, i32, i32, i32, vp, vp, vp],
            "pt_zero_groups_batched": [C.POINTER(NormMask), i32, f32, vp],
            "pt_reconcile_plan_batched": [C.POINTER(EdgePlan), i32, vp],
            "pt_compact_vector_batched": [C.POINTER(GatherVector), i32, vp],
            "pt_compact_weights_batched": [C.POINTER(GatherWeights), i32, vp],
            "pt_plan_layer_removal": [C.POINTER(RemovalEdge), i32, i32, vp, vp],
            "pt_conv_fwd_stats_workspace_bytes": [dp, C.POINTER(sz), C.POINTER(i32)],
            "pt_conv_fwd_stats": [dp, vp, vp, vp, vp, sz, vp],
            "pt_bn_fwd_from_sums": [vp, i64, i32, i32, vp, i32, vp, vp, f32, vp, i32, vp, vp, vp],
            "pt_bn_workspace_bytes": [i64, i32, C.POINTER(sz)],
            "pt_bn_fwd": [vp, i64, i32, i32, vp, vp, f32, vp, i32, vp, vp, vp, sz, vp],
            "pt_bn_bwd": [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp],
        }
        for name, args in sig.items():
            fn = getattr(_lib, name)
            fn.argtypes = args
            fn.restype = i32
    return _lib


def _ck(name: str, rc: int) -> None:
    if rc != PT_OK:
        raise PruneTrainError(name, rc)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def conv_desc(N, H, W, Cc, K, R, S, stride, pad, x_cpitch=None, y_cpitch=None, w_cpitch=None, flags=0) -> ConvDesc:
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    return ConvDesc(C.sizeof(ConvDesc), N, H, W, Cc, K, R, S, stride, stride, pad, pad, P, Q,
                    x_cpitch or Cc, y_cpitch or K, w_cpitch or Cc, flags)


def desc_of(spec, x_cpitch=None, y_cpitch=None, w_cpitch=None, flags=0) -> ConvDesc:
    return conv_desc(spec.N, spec.H, spec.W, spec.C, spec.K, spec.R, spec.S, spec.stride, spec.pad,
                     x_cpitch, y_cpitch, w_cpitch, flags)


def version() -> int:
    return lib().pt_version()


def _ws_bytes(fn: str, d: ConvDesc) -> int:
    n = C.c_size_t(0)
    _ck(fn, getattr(lib(), fn)(C.byref(d), C.byref(n)))
    return n.value


def conv_fwd_workspace_bytes(d: ConvDesc) -> int:
    return _ws_bytes("pt_conv_fwd_workspace_bytes", d)


def conv_bwd_data_workspace_bytes(d: ConvDesc) -> int:
    return _ws_bytes("pt_conv_bwd_data_workspace_bytes", d)


def conv_bwd_weight_workspace_bytes(d: ConvDesc) -> int:
    return _ws_bytes("pt_conv_bwd_weight_workspace_bytes", d)


def _ws(ws):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


def conv_fwd(d: ConvDesc, x, w, y, ws=None, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_conv_fwd", lib().pt_conv_fwd(C.byref(d), _ptr(x), _ptr(w), _ptr(y), p, n, _stream(stream)))


def conv_fwd_jobs(descs: Sequence[ConvDesc], xs, ws, ys):
    """Argument arrays of conv_fwd_batched, built once for a fixed set of layers."""
    n = len(descs)
    return ((ConvDesc * n)(*descs), (C.c_void_p * n)(*[_ptr(t) for t in xs]), (C.c_void_p * n)(*[_ptr(t) for t in ws]),
            (C.c_void_p * n)(*[_ptr(t) for t in ys]), n)


def conv_fwd_batched(jobs, stream=None) -> None:
    d, x, w, y, n = jobs
    _ck("pt_conv_fwd_batched", lib().pt_conv_fwd_batched(d, x, w, y, n, _stream(stream)))


def conv_bwd_data(d: ConvDesc, dy, w, dx, ws=None, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_conv_bwd_data", lib().pt_conv_bwd_data(C.byref(d), _ptr(dy), _ptr(w), _ptr(dx), p, n, _stream(stream)))


def conv_bwd_weight(d: ConvDesc, x, dy, dw, ws=None, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_conv_bwd_weight",
        lib().pt_conv_bwd_weight(C.byref(d), _ptr(x), _ptr(dy), _ptr(dw), p, n, _stream(stream)))


def conv_bwd_weight_lasso_workspace_bytes(d: ConvDesc) -> int:
    return _ws_bytes("pt_conv_bwd_weight_lasso_workspace_bytes", d)


def conv_bwd_weight_lasso(d: ConvDesc, x, dy, w, out_norm, in_norm, lam: float, flags: int, dw, ws=None, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_conv_bwd_weight_lasso",
        lib().pt_conv_bwd_weight_lasso(C.byref(d), _ptr(x), _ptr(dy), _ptr(w), _ptr(out_norm), _ptr(in_norm), lam, flags,
                                       _ptr(dw), p, n, _stream(stream)))


def group_norms_workspace_bytes(K: int, RS: int, Cc: int) -> int:
    n = C.c_size_t(0)
    _ck("pt_group_norms_workspace_bytes", lib().pt_group_norms_workspace_bytes(K, RS, Cc, C.byref(n)))
    return n.value


def group_norms(w, K, RS, Cc, w_cpitch, out_norm, in_norm, w_shadow=None, ws=None, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_group_norms", lib().pt_group_norms(_ptr(w), K, RS, Cc, w_cpitch, _ptr(out_norm), _ptr(in_norm),
                                               _ptr(w_shadow), p, n, _stream(stream)))


def group_lasso_grad(w, out_norm, in_norm, lam: float, flags: int, dw, K, RS, Cc, w_cpitch, stream=None) -> None:
    _ck("pt_group_lasso_grad", lib().pt_group_lasso_grad(_ptr(w), _ptr(out_norm), _ptr(in_norm), lam, flags, _ptr(dw),
                                                         K, RS, Cc, w_cpitch, _stream(stream)))


def group_norms_static(w, K: int, RS: int, Cc: int, w_cpitch: int, out_norm, in_norm, w_shadow=None, stream=None) -> None:
    """pt_group_norms without a workspace argument: the library's own per-device scratch is used."""
    _ck("pt_group_norms_static", lib().pt_group_norms_static(_ptr(w), K, RS, Cc, w_cpitch, _ptr(out_norm), _ptr(in_norm),
                                                            _ptr(w_shadow), _stream(stream)))


def layer_weights(w, K, RS, Cc, w_cpitch, out_norm, in_norm, w_shadow=None) -> LayerWeights:
    return LayerWeights(_ptr(w), _ptr(out_norm), _ptr(in_norm), _ptr(w_shadow), K, RS, Cc, w_cpitch)


def layer_lasso(w, out_norm, in_norm, dw, K, RS, Cc, w_cpitch, flags) -> LayerLasso:
    return LayerLasso(_ptr(w), _ptr(out_norm), _ptr(in_norm), _ptr(dw), K, RS, Cc, w_cpitch, flags, 0)


def _array(items, typ):
    return items if isinstance(items, C.Array) else (typ * max(1, len(items)))(*items)


def group_norms_batched_workspace_bytes(layers) -> int:
    arr = _array(layers, LayerWeights)
    n = C.c_size_t(0)
    _ck("pt_group_norms_batched_workspace_bytes", lib().pt_group_norms_batched_workspace_bytes(arr, len(layers), C.byref(n)))
    return n.value


def group_norms_batched(layers, ws, stream=None) -> None:
    """layers: list of LayerWeights (or a prepared ctypes array of them)."""
    arr = _array(layers, LayerWeights)
    p, n = _ws(ws)
    _ck("pt_group_norms_batched", lib().pt_group_norms_batched(arr, len(layers), p, n, _stream(stream)))


def layer_detect(w, K, RS, Cc, w_cpitch, out_norm, in_norm, zero_out, zero_in) -> LayerDetect:
    return LayerDetect(_ptr(w), _ptr(out_norm), _ptr(in_norm), _ptr(zero_out), _ptr(zero_in), K, RS, Cc, w_cpitch)


def group_norms_detect_batched_workspace_bytes(layers) -> int:
    arr = _array(layers, LayerDetect)
    n = C.c_size_t(0)
    _ck("pt_group_norms_detect_batched_workspace_bytes",
        lib().pt_group_norms_detect_batched_workspace_bytes(arr, len(layers), C.byref(n)))
    return n.value


def group_norms_detect_batched(layers, thr: float, ws, stream=None) -> None:
    """layers: list of LayerDetect (or a prepared ctypes array): norms and zero masks of every layer."""
    arr = _array(layers, LayerDetect)
    p, n = _ws(ws)
    _ck("pt_group_norms_detect_batched", lib().pt_group_norms_detect_batched(arr, len(layers), thr, p, n, _stream(stream)))


def conv_bwd_weight_plan(d: ConvDesc, aligned: bool = True) -> WgradPlanInfo:
    info = WgradPlanInfo()
    _ck("pt_conv_bwd_weight_plan", lib().pt_conv_bwd_weight_plan(C.byref(d), 1 if aligned else 0, C.byref(info)))
    return info


def group_lasso_grad_batched(layers, lam: float, stream=None) -> None:
    arr = _array(layers, LayerLasso)
    _ck("pt_group_lasso_grad_batched", lib().pt_group_lasso_grad_batched(arr, len(layers), lam, _stream(stream)))


def zero_groups(norms, n: int, thr: float, zero, stream=None) -> None:
    _ck("pt_zero_groups", lib().pt_zero_groups(_ptr(norms), n, thr, _ptr(zero), _stream(stream)))


def reconcile_edge(producer_zero: Sequence, consumer_zero: Sequence, n: int, keep, stream=None) -> None:
    pa = (C.c_void_p * max(1, len(producer_zero)))(*[t.data_ptr() for t in producer_zero])
    ca = (C.c_void_p * max(1, len(consumer_zero)))(*[t.data_ptr() for t in consumer_zero])
    _ck("pt_reconcile_edge", lib().pt_reconcile_edge(pa if len(producer_zero) else None, len(producer_zero),
                                                     ca if len(consumer_zero) else None, len(consumer_zero), n,
                                                     _ptr(keep), _stream(stream)))


def compact_plan(keep, n: int, idx, n_keep_dev, stream=None) -> None:
    _ck("pt_compact_plan", lib().pt_compact_plan(_ptr(keep), n, _ptr(idx), _ptr(n_keep_dev), _stream(stream)))


def compact_weights(w, K, RS, Cc, w_cpitch, idxK, Kp, idxC, Cp, w_out, out_cpitch, stream=None) -> None:
    _ck("pt_compact_weights", lib().pt_compact_weights(_ptr(w), K, RS, Cc, w_cpitch, _ptr(idxK), Kp, _ptr(idxC), Cp,
                                                       _ptr(w_out), out_cpitch, _stream(stream)))


def compact_vector(v, elem_bytes: int, idx, n_keep: int, out, stream=None) -> None:
    _ck("pt_compact_vector", lib().pt_compact_vector(_ptr(v), elem_bytes, _ptr(idx), n_keep, _ptr(out),
                                                     _stream(stream)))


def compact_nhwc(x, pixels: int, Cc: int, x_cpitch: int, idx, Cp: int, out, out_cpitch: int, stream=None) -> None:
    _ck("pt_compact_nhwc", lib().pt_compact_nhwc(_ptr(x), pixels, Cc, x_cpitch, _ptr(idx), Cp, _ptr(out), out_cpitch,
                                                 _stream(stream)))


# ---- multi-job forms ------------------------------------------------------------------------------ #
def norm_mask(norms, n: int, zero) -> NormMask:
    return NormMask(_ptr(norms), _ptr(zero), n, 0)


def zero_groups_batched(jobs, thr: float, stream=None) -> None:
    arr = _array(jobs, NormMask)
    _ck("pt_zero_groups_batched", lib().pt_zero_groups_batched(arr, len(jobs), thr, _stream(stream)))


def edge_plan(producer_zero: Sequence, consumer_zero: Sequence, n: int, keep, idx, n_keep_dev) -> EdgePlan:
    """The member pointer arrays are host arrays owned by the returned struct (kept alive with it)."""
    pa = (C.c_void_p * max(1, len(producer_zero)))(*[t.data_ptr() for t in producer_zero])
    ca = (C.c_void_p * max(1, len(consumer_zero)))(*[t.data_ptr() for t in consumer_zero])
    e = EdgePlan(C.cast(pa, C.POINTER(C.c_void_p)) if len(producer_zero) else None,
                 C.cast(ca, C.POINTER(C.c_void_p)) if len(consumer_zero) else None,
                 len(producer_zero), len(consumer_zero), n, 0, _ptr(keep), _ptr(idx), _ptr(n_keep_dev))
    e._keepalive = (pa, ca)
    return e


def reconcile_plan_batched(edges, stream=None) -> None:
    arr = _array(edges, EdgePlan)
    _ck("pt_reconcile_plan_batched", lib().pt_reconcile_plan_batched(arr, len(edges), _stream(stream)))


def gather_vector(v, elem_bytes: int, idx, n_keep: int, out) -> GatherVector:
    return GatherVector(_ptr(v), _ptr(idx), _ptr(out), n_keep, elem_bytes)


def compact_vector_batched(jobs, stream=None) -> None:
    arr = _array(jobs, GatherVector)
    _ck("pt_compact_vector_batched", lib().pt_compact_vector_batched(arr, len(jobs), _stream(stream)))


def gather_weights(w, K, RS, Cc, w_cpitch, idxK, Kp, idxC, Cp, w_out, out_cpitch) -> GatherWeights:
    return GatherWeights(_ptr(w), _ptr(idxK), _ptr(idxC), _ptr(w_out), K, RS, Cc, w_cpitch, Kp, Cp, out_cpitch, 0)


def compact_weights_batched(jobs, stream=None) -> None:
    arr = _array(jobs, GatherWeights)
    _ck("pt_compact_weights_batched", lib().pt_compact_weights_batched(arr, len(jobs), _stream(stream)))


def layer_crsk(w, wt, K, RS, Cc, w_cpitch) -> LayerCrsk:
    return LayerCrsk(_ptr(w), _ptr(wt), K, RS, Cc, w_cpitch)


def weights_to_crsk_batched(layers, stream=None) -> None:
    arr = _array(layers, LayerCrsk)
    _ck("pt_weights_to_crsk_batched", lib().pt_weights_to_crsk_batched(arr, len(layers), _stream(stream)))


def conv_bwd_data_crsk(d: ConvDesc, dy, wt, dx, stream=None) -> None:
    _ck("pt_conv_bwd_data_crsk", lib().pt_conv_bwd_data_crsk(C.byref(d), _ptr(dy), _ptr(wt), _ptr(dx), _stream(stream)))


def layer_penalty(out_norm, in_norm, K: int, Cc: int, flags: int) -> LayerPenalty:
    return LayerPenalty(_ptr(out_norm), _ptr(in_norm), K, Cc, flags, 0)


def group_lasso_penalty_batched(layers, penalty_dev, stream=None) -> None:
    """penalty_dev: a float64 device tensor with one element."""
    arr = _array(layers, LayerPenalty)
    _ck("pt_group_lasso_penalty_batched",
        lib().pt_group_lasso_penalty_batched(arr, len(layers), _ptr(penalty_dev), _stream(stream)))


def lasso_set_coeff(loss1: float, loss2: float, ratio: float) -> float:
    lam = C.c_double(0.0)
    _ck("pt_lasso_set_coeff", lib().pt_lasso_set_coeff(loss1, loss2, ratio, C.byref(lam)))
    return lam.value


def gather_nhwc(x, pixels: int, Cc: int, x_cpitch: int, idx, Cp: int, out, out_cpitch: int) -> GatherNhwc:
    return GatherNhwc(_ptr(x), _ptr(idx), _ptr(out), pixels, Cc, x_cpitch, Cp, out_cpitch)


def compact_nhwc_batched(jobs, stream=None) -> None:
    arr = _array(jobs, GatherNhwc)
    _ck("pt_compact_nhwc_batched", lib().pt_compact_nhwc_batched(arr, len(jobs), _stream(stream)))


def scatter_nhwc(x, pixels: int, Cp: int, x_cpitch: int, idx, Cc: int, out, out_cpitch: int, stream=None) -> None:
    _ck("pt_scatter_nhwc", lib().pt_scatter_nhwc(_ptr(x), pixels, Cp, x_cpitch, _ptr(idx), Cc, _ptr(out), out_cpitch,
                                                 _stream(stream)))


def group_maxabs(w, K, RS, Cc, w_cpitch, out_max, in_max, stream=None) -> None:
    _ck("pt_group_maxabs", lib().pt_group_maxabs(_ptr(w), K, RS, Cc, w_cpitch, _ptr(out_max), _ptr(in_max),
                                                 _stream(stream)))


def apply_zero(w, K, RS, Cc, w_cpitch, zero_out=None, zero_in=None, stream=None) -> None:
    _ck("pt_apply_zero", lib().pt_apply_zero(_ptr(w), K, RS, Cc, w_cpitch, _ptr(zero_out), _ptr(zero_in),
                                             _stream(stream)))


def layer_update(w, dw, mom, out_norm, in_norm, K, RS, Cc, w_cpitch, flags) -> LayerUpdate:
    return LayerUpdate(_ptr(w), _ptr(dw), _ptr(mom), _ptr(out_norm), _ptr(in_norm), K, RS, Cc, w_cpitch, flags, 0)


def sgd_momentum_lasso_batched(layers, lam: float, lr: float, momentum: float, weight_decay: float, stream=None) -> None:
    arr = _array(layers, LayerUpdate)
    _ck("pt_sgd_momentum_lasso_batched",
        lib().pt_sgd_momentum_lasso_batched(arr, len(layers), lam, lr, momentum, weight_decay, _stream(stream)))


def bn_workspace_bytes(pixels: int, Cc: int) -> int:
    n = C.c_size_t(0)
    _ck("pt_bn_workspace_bytes", lib().pt_bn_workspace_bytes(pixels, Cc, C.byref(n)))
    return n.value


def bn_fwd(x, pixels: int, Cc: int, x_cpitch: int, gamma, beta, eps: float, y, y_cpitch: int, mean, invstd, ws,
           stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_bn_fwd", lib().pt_bn_fwd(_ptr(x), pixels, Cc, x_cpitch, _ptr(gamma), _ptr(beta), eps, _ptr(y), y_cpitch,
                                     _ptr(mean), _ptr(invstd), p, n, _stream(stream)))


def bn_bwd(x, dy, pixels: int, Cc: int, x_cpitch: int, dy_cpitch: int, gamma, mean, invstd, dx, dx_cpitch: int,
           dgamma, dbeta, ws, stream=None) -> None:
    p, n = _ws(ws)
    _ck("pt_bn_bwd", lib().pt_bn_bwd(_ptr(x), _ptr(dy), pixels, Cc, x_cpitch, dy_cpitch, _ptr(gamma), _ptr(mean),
                                     _ptr(invstd), _ptr(dx), dx_cpitch, _ptr(dgamma), _ptr(dbeta), p, n,
                                     _stream(stream)))


def plan_layer_removal(edges: Sequence, n_layers: int):
    """edges: (producers, consumers, n_keep, external) per edge, all host values.  Returns (removed_layers,
    dead_edges, status) as lists of 0/1 and the call's status (PT_OK, or PT_ERR_EMPTY when the network is cut)."""
    keep_alive = []
    arr = (RemovalEdge * max(1, len(edges)))()
    for i, (prod, cons, n_keep, external) in enumerate(edges):
        p, c = (C.c_int32 * max(1, len(prod)))(*prod), (C.c_int32 * max(1, len(cons)))(*cons)
        keep_alive += [p, c]
        arr[i] = RemovalEdge(p, c, len(prod), len(cons), n_keep, external)
    removed, dead = (C.c_uint8 * max(1, n_layers))(), (C.c_uint8 * max(1, len(edges)))()
    rc = lib().pt_plan_layer_removal(arr, len(edges), n_layers, removed, dead)
    if rc not in (PT_OK, -6):
        raise PruneTrainError("pt_plan_layer_removal", rc)
    return list(removed)[:n_layers], list(dead)[:len(edges)], rc


def conv_fwd_stats_workspace(d: ConvDesc):
    """-> (bytes of the sums buffer, number of partial rows per statistic)."""
    n, k = C.c_size_t(0), C.c_int32(0)
    _ck("pt_conv_fwd_stats_workspace_bytes", lib().pt_conv_fwd_stats_workspace_bytes(C.byref(d), C.byref(n), C.byref(k)))
    return n.value, k.value


def conv_fwd_stats(d: ConvDesc, x, w, y, sums, stream=None) -> None:
    p, n = _ws(sums)
    _ck("pt_conv_fwd_stats", lib().pt_conv_fwd_stats(C.byref(d), _ptr(x), _ptr(w), _ptr(y), p, n, _stream(stream)))


def bn_fwd_from_sums(x, pixels: int, Cc: int, x_cpitch: int, sums, n_partial: int, gamma, beta, eps: float, y,
                     y_cpitch: int, mean, invstd, stream=None) -> None:
    _ck("pt_bn_fwd_from_sums", lib().pt_bn_fwd_from_sums(_ptr(x), pixels, Cc, x_cpitch, _ptr(sums), n_partial, _ptr(gamma),
                                                         _ptr(beta), eps, _ptr(y), y_cpitch, _ptr(mean), _ptr(invstd),
                                                         _stream(stream)))
