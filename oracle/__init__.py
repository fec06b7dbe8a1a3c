"""ctypes front end of the fp64 CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg; the product package never imports it and it never
imports the product package.  numpy in, numpy out, everything promoted to fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (-O2, OpenMP) into liboracle.so next to the source."""
    src = os.path.join(_HERE, "oracle.c")
    hdr = os.path.join(_HERE, "oracle.h")
    if (not force and os.path.exists(_SO)
            and os.path.getmtime(_SO) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _SO
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _SO, src, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


class ConvShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "P", "Q")]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        for name in ("oracle_num_threads",):
            getattr(_lib, name).restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(C.c_int(n))


def shape(N, H, W, Cc, K, R, S, stride, pad, P=None, Q=None) -> ConvShape:
    sh = sw = stride
    ph = pw = pad
    if P is None:
        P = (H + 2 * ph - R) // sh + 1
    if Q is None:
        Q = (W + 2 * pw - S) // sw + 1
    return ConvShape(N, H, W, Cc, K, R, S, sh, sw, ph, pw, P, Q)


def shape_of(spec) -> ConvShape:
    """ConvShape of anything with N,H,W,C,K,R,S,stride,pad attributes."""
    return shape(spec.N, spec.H, spec.W, spec.C, spec.K, spec.R, spec.S, spec.stride, spec.pad)


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what}: oracle status {rc}")


def conv_fwd(s: ConvShape, x, w) -> np.ndarray:
    x, w = _d(x), _d(w)
    assert x.size == s.N * s.H * s.W * s.C and w.size == s.K * s.R * s.S * s.C
    y = np.empty((s.N, s.P, s.Q, s.K), dtype=np.float64)
    _check(_load().oracle_conv_fwd(C.byref(s), _p(x), _p(w), _p(y)), "conv_fwd")
    return y


def conv_bwd_data(s: ConvShape, dy, w) -> np.ndarray:
    dy, w = _d(dy), _d(w)
    assert dy.size == s.N * s.P * s.Q * s.K and w.size == s.K * s.R * s.S * s.C
    dx = np.empty((s.N, s.H, s.W, s.C), dtype=np.float64)
    _check(_load().oracle_conv_bwd_data(C.byref(s), _p(dy), _p(w), _p(dx)), "conv_bwd_data")
    return dx


def conv_bwd_weight(s: ConvShape, x, dy) -> np.ndarray:
    x, dy = _d(x), _d(dy)
    assert x.size == s.N * s.H * s.W * s.C and dy.size == s.N * s.P * s.Q * s.K
    dw = np.empty((s.K, s.R, s.S, s.C), dtype=np.float64)
    _check(_load().oracle_conv_bwd_weight(C.byref(s), _p(x), _p(dy), _p(dw)), "conv_bwd_weight")
    return dw


def _at(fn_name: str, s: ConvShape, a, b, idx) -> np.ndarray:
    a, b = _d(a), _d(b)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    fn = getattr(_load(), fn_name)
    _check(fn(C.byref(s), _p(a), _p(b), _p(idx), C.c_int64(idx.size), _p(out)), fn_name)
    return out


def conv_fwd_at(s, x, w, idx):
    assert np.size(x) == s.N * s.H * s.W * s.C and np.size(w) == s.K * s.R * s.S * s.C
    return _at("oracle_conv_fwd_at", s, x, w, idx)


def conv_bwd_data_at(s, dy, w, idx):
    assert np.size(dy) == s.N * s.P * s.Q * s.K and np.size(w) == s.K * s.R * s.S * s.C
    return _at("oracle_conv_bwd_data_at", s, dy, w, idx)


def conv_bwd_weight_at(s, x, dy, idx):
    assert np.size(x) == s.N * s.H * s.W * s.C and np.size(dy) == s.N * s.P * s.Q * s.K
    return _at("oracle_conv_bwd_weight_at", s, x, dy, idx)


def group_norms(w):
    """w [K,R,S,C] (or [K,RS,C]) -> (out_norm[K], in_norm[C])."""
    w = _d(w)
    K, Cc = w.shape[0], w.shape[-1]
    RS = w.size // (K * Cc)
    on = np.empty(K, dtype=np.float64)
    inn = np.empty(Cc, dtype=np.float64)
    _check(_load().oracle_group_norms(_p(w), K, RS, Cc, _p(on), _p(inn)), "group_norms")
    return on, inn


def group_lasso_grad(w, out_norm, in_norm, lam: float, flags: int, dw) -> np.ndarray:
    """Returns dw + gradient of lam * (sum out_norm + sum in_norm); dw is not modified."""
    w = _d(w)
    K, Cc = w.shape[0], w.shape[-1]
    RS = w.size // (K * Cc)
    on, inn = _d(out_norm), _d(in_norm)
    assert on.size == K and inn.size == Cc
    g = _d(dw).copy()
    assert g.size == w.size
    _check(_load().oracle_group_lasso_grad(_p(w), _p(on), _p(inn), C.c_double(lam), C.c_uint32(flags), _p(g),
                                           K, RS, Cc), "group_lasso_grad")
    return g.reshape(w.shape)


def group_lasso_penalty(layers) -> float:
    """layers: iterable of (out_norm, in_norm, flags); the regulariser's value summed over them."""
    p = C.c_double(0.0)
    for on, inn, flags in layers:
        on, inn = _d(on), _d(inn)
        _check(_load().oracle_group_lasso_penalty(_p(on), on.size, _p(inn), inn.size, C.c_uint32(flags), C.byref(p)),
               "group_lasso_penalty")
    return p.value


def set_coeff(loss1: float, loss2: float, ratio: float) -> float:
    lam = C.c_double(0.0)
    _check(_load().oracle_set_coeff(C.c_double(loss1), C.c_double(loss2), C.c_double(ratio), C.byref(lam)), "set_coeff")
    return lam.value


def zero_groups(norms, thr: float) -> np.ndarray:
    norms = _d(norms)
    z = np.empty(norms.size, dtype=np.uint8)
    _check(_load().oracle_zero_groups(_p(norms), norms.size, C.c_double(thr), _p(z)), "zero_groups")
    return z


def reconcile_edge(producer_zero: Sequence[np.ndarray], consumer_zero: Sequence[np.ndarray]) -> np.ndarray:
    prods = [np.ascontiguousarray(a, dtype=np.uint8) for a in producer_zero]
    cons = [np.ascontiguousarray(a, dtype=np.uint8) for a in consumer_zero]
    n = (prods + cons)[0].size
    assert all(a.size == n for a in prods + cons)
    PA = (C.c_void_p * max(1, len(prods)))(*[a.ctypes.data for a in prods])
    CA = (C.c_void_p * max(1, len(cons)))(*[a.ctypes.data for a in cons])
    keep = np.empty(n, dtype=np.uint8)
    _check(_load().oracle_reconcile_edge(PA if prods else None, len(prods), CA if cons else None, len(cons), n,
                                         _p(keep)), "reconcile_edge")
    return keep


def compact_plan(keep) -> np.ndarray:
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    idx = np.empty(keep.size, dtype=np.int32)
    nk = C.c_int32(0)
    _check(_load().oracle_compact_plan(_p(keep), keep.size, _p(idx), C.byref(nk)), "compact_plan")
    return idx[: nk.value].copy()


def compact_weights(w, idxK: Optional[np.ndarray], idxC: Optional[np.ndarray]) -> np.ndarray:
    w = _d(w)
    K, Cc = w.shape[0], w.shape[-1]
    RS = w.size // (K * Cc)
    ik = None if idxK is None else np.ascontiguousarray(idxK, dtype=np.int32)
    ic = None if idxC is None else np.ascontiguousarray(idxC, dtype=np.int32)
    Kp = K if ik is None else ik.size
    Cp = Cc if ic is None else ic.size
    out = np.empty((Kp,) + tuple(w.shape[1:-1]) + (Cp,), dtype=np.float64)
    _check(_load().oracle_compact_weights(_p(w), K, RS, Cc, None if ik is None else _p(ik), Kp,
                                          None if ic is None else _p(ic), Cp, _p(out)), "compact_weights")
    return out


def compact_vector(v, idx) -> np.ndarray:
    v = np.ascontiguousarray(v)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < v.size)
    out = np.empty(idx.size, dtype=v.dtype)
    _check(_load().oracle_compact_vector(_p(v), v.dtype.itemsize, _p(idx), idx.size, _p(out)), "compact_vector")
    return out


def compact_nhwc(x, idx) -> np.ndarray:
    """x [..., C] of any fixed-size dtype -> x[..., idx], copied byte for byte."""
    x = np.ascontiguousarray(x)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Cc = x.shape[-1]
    pixels = x.size // Cc
    out = np.empty(x.shape[:-1] + (idx.size,), dtype=x.dtype)
    _check(_load().oracle_compact_nhwc(_p(x), C.c_int64(pixels), Cc, x.dtype.itemsize, _p(idx), idx.size, _p(out)),
           "compact_nhwc")
    return out


def scatter_nhwc(x, idx, Cc: int) -> np.ndarray:
    """x [..., Cp] -> out [..., Cc] with out[..., idx] = x and zeros elsewhere (byte-exact copy)."""
    x = np.ascontiguousarray(x)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Cp = x.shape[-1]
    assert idx.size == Cp
    pixels = x.size // Cp
    out = np.empty(x.shape[:-1] + (Cc,), dtype=x.dtype)
    _check(_load().oracle_scatter_nhwc(_p(x), C.c_int64(pixels), Cp, x.dtype.itemsize, _p(idx), Cc, _p(out)),
           "scatter_nhwc")
    return out


def group_maxabs(w):
    """w [K,R,S,C] -> (out_max[K], in_max[C])."""
    w = _d(w)
    K, Cc = w.shape[0], w.shape[-1]
    RS = w.size // (K * Cc)
    om = np.empty(K, dtype=np.float64)
    im = np.empty(Cc, dtype=np.float64)
    _check(_load().oracle_group_maxabs(_p(w), K, RS, Cc, _p(om), _p(im)), "group_maxabs")
    return om, im


def apply_zero(w, zero_out=None, zero_in=None) -> np.ndarray:
    """Returns a copy of w with the flagged groups written to exact zero."""
    out = _d(w).copy()
    K, Cc = out.shape[0], out.shape[-1]
    RS = out.size // (K * Cc)
    zo = None if zero_out is None else np.ascontiguousarray(zero_out, dtype=np.uint8)
    zi = None if zero_in is None else np.ascontiguousarray(zero_in, dtype=np.uint8)
    assert (zo is None or zo.size == K) and (zi is None or zi.size == Cc)
    _check(_load().oracle_apply_zero(_p(out), K, RS, Cc, None if zo is None else _p(zo), None if zi is None else _p(zi)),
           "apply_zero")
    return out


def sgd_momentum_lasso(w, dw, mom, out_norm, in_norm, lam, lr, mu, wd, flags):
    """Returns (w_new, mom_new); inputs are not modified."""
    w2, m2, g = _d(w).copy(), _d(mom).copy(), _d(dw)
    K, Cc = w2.shape[0], w2.shape[-1]
    RS = w2.size // (K * Cc)
    on, inn = _d(out_norm), _d(in_norm)
    assert g.size == w2.size and m2.size == w2.size and on.size == K and inn.size == Cc
    _check(_load().oracle_sgd_momentum_lasso(_p(w2), _p(g), _p(m2), _p(on), _p(inn), C.c_double(lam), C.c_double(lr),
                                             C.c_double(mu), C.c_double(wd), C.c_uint32(flags), K, RS, Cc),
           "sgd_momentum_lasso")
    return w2, m2


def bn_fwd(x, gamma, beta, eps: float):
    """x [..., C] -> (y, mean[C], invstd[C]) with batch statistics over all leading axes."""
    x = _d(x)
    Cc = x.shape[-1]
    pixels = x.size // Cc
    g, b = _d(gamma), _d(beta)
    assert g.size == Cc and b.size == Cc
    y = np.empty_like(x)
    mean = np.empty(Cc, dtype=np.float64)
    invstd = np.empty(Cc, dtype=np.float64)
    _check(_load().oracle_bn_fwd(_p(x), C.c_int64(pixels), Cc, _p(g), _p(b), C.c_double(eps), _p(y), _p(mean), _p(invstd)),
           "bn_fwd")
    return y, mean, invstd


def bn_bwd(x, dy, gamma, mean, invstd):
    """-> (dx, dgamma[C], dbeta[C])."""
    x, dy = _d(x), _d(dy)
    Cc = x.shape[-1]
    pixels = x.size // Cc
    g, m, s = _d(gamma), _d(mean), _d(invstd)
    dx = np.empty_like(x)
    dg = np.empty(Cc, dtype=np.float64)
    db = np.empty(Cc, dtype=np.float64)
    _check(_load().oracle_bn_bwd(_p(x), _p(dy), C.c_int64(pixels), Cc, _p(g), _p(m), _p(s), _p(dx), _p(dg), _p(db)),
           "bn_bwd")
    return dx, dg, db


def plan_layer_removal(n_layers: int, edges):
    """Layer removal after a plan (Sec. 4.1, "Layer Removal by Overlapping Regularization Groups"), as sets.

    edges: one (producers, consumers, n_keep, fed_outside, read_outside) per channel edge.  An edge with no
    survivors carries nothing, so the layers on either side of it go; an edge whose listed producers are all
    gone (and that nothing outside feeds) carries nothing, one whose listed consumers are all gone (and that
    nothing outside reads) is read by nobody.  Iterated to the fixed point.  Returns (removed layer set, dead
    edge set, cut) where cut says that an edge read outside the listed layers has died."""
    dead = {e for e, ed in enumerate(edges) if ed[2] == 0}
    removed = set()
    while True:
        new_removed = set(removed)
        for e in dead:
            new_removed |= set(edges[e][0]) | set(edges[e][1])
        new_dead = set(dead)
        for e, (prod, cons, _, fed_outside, read_outside) in enumerate(edges):
            starved = len(prod) > 0 and not fed_outside and set(prod) <= new_removed
            unread = len(cons) > 0 and not read_outside and set(cons) <= new_removed
            if starved or unread:
                new_dead.add(e)
        if new_removed == removed and new_dead == dead:
            break
        removed, dead = new_removed, new_dead
    assert all(0 <= l < n_layers for l in removed)
    cut = any(edges[e][4] for e in dead)
    return removed, dead, cut
