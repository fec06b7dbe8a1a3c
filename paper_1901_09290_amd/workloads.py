"""Seeded synthetic workloads: layer tables, channel edges and random tensors.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
convolution, no norm, no mask logic, no gather): both the HIP path and the CPU
oracle are fed from here and neither is imported here.

Shapes follow the networks the paper trains (ResNet-32 on CIFAR-sized images,
ResNet-50 on ImageNet-sized images; Evaluation Methodology section).  The
datasets themselves are not used: activations and upstream gradients are
N(0,1), weights are He-normal with std = sqrt(2 / (R*S*C)).

Conventions: activations NHWC, weights K,R,S,C (output channel, filter row,
filter column, input channel).  A *channel edge* is a set of convolutions whose
output dimension (producers) and input dimension (consumers) must stay equal
after pruning: one producer and one consumer for a plain edge, every conv that
touches the shared node for a residual stage.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------- #
# bf16 value grid helpers (input quantisation only)
# --------------------------------------------------------------------------- #
def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable fp32 (ties to even)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that already lie on the bf16 grid."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not on the bf16 grid"
    return (u >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """fp32 values of uint16 bf16 bit patterns."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# layer tables
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class ConvSpec:
    name: str
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    in_edge: Optional[int]   # edge id of the input channel dimension (None: image)
    out_edge: Optional[int]  # edge id of the output channel dimension
    first: bool = False      # network's first conv: no bwd_data, input groups exempt

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def flops(self) -> int:
        """2*N*P*Q*K*C*R*S: one pass (fwd, bwd_data or bwd_weight)."""
        return 2 * self.N * self.P * self.Q * self.K * self.C * self.R * self.S

    @property
    def params(self) -> int:
        return self.K * self.R * self.S * self.C

    def shape_key(self) -> Tuple[int, ...]:
        return (self.N, self.H, self.W, self.C, self.K, self.R, self.S, self.stride, self.pad)


@dataclass
class Edge:
    name: str
    n: int
    producers: List[int] = field(default_factory=list)  # layer indices (output dim)
    consumers: List[int] = field(default_factory=list)  # layer indices (input dim)


def _link(layers: List[ConvSpec], edges: List[Edge]) -> None:
    for e in edges:
        e.producers.clear()
        e.consumers.clear()
    for i, l in enumerate(layers):
        if l.out_edge is not None:
            edges[l.out_edge].producers.append(i)
        if l.in_edge is not None:
            edges[l.in_edge].consumers.append(i)


def resnet50_layers(N: int = 64, image: int = 224) -> Tuple[List[ConvSpec], List[Edge]]:
    """The 53 convolutions of ResNet-50 (stride on the 3x3, 1x1 projections).

    Edges: stem output, four stage nodes, two private edges per bottleneck.
    """
    layers: List[ConvSpec] = []
    edges: List[Edge] = []

    def new_edge(name: str, n: int) -> int:
        edges.append(Edge(name, n))
        return len(edges) - 1

    e_stem = new_edge("stem_out", 64)
    layers.append(ConvSpec("stem", N, image, image, 3, 64, 7, 7, 2, 3, None, e_stem, first=True))
    h = (image + 2 * 3 - 7) // 2 + 1          # 112
    h = (h + 2 * 1 - 3) // 2 + 1              # max-pool 3x3 s2 p1 -> 56 (not a conv)
    node_in, c_in = e_stem, 64
    for si, (width, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)]):
        stage = si + 2
        c_out = 4 * width
        node = new_edge(f"conv{stage}_node", c_out)
        for b in range(blocks):
            st = 2 if (b == 0 and stage > 2) else 1
            src, c_src = (node_in, c_in) if b == 0 else (node, c_out)
            ea = new_edge(f"conv{stage}_b{b}_a", width)
            eb = new_edge(f"conv{stage}_b{b}_b", width)
            layers.append(ConvSpec(f"conv{stage}_b{b}_1x1a", N, h, h, c_src, width, 1, 1, 1, 0, src, ea))
            layers.append(ConvSpec(f"conv{stage}_b{b}_3x3", N, h, h, width, width, 3, 3, st, 1, ea, eb))
            ho = h // st
            layers.append(ConvSpec(f"conv{stage}_b{b}_1x1b", N, ho, ho, width, c_out, 1, 1, 1, 0, eb, node))
            if b == 0:
                layers.append(ConvSpec(f"conv{stage}_proj", N, h, h, c_src, c_out, 1, 1, st, 0, src, node))
            h = ho
        node_in, c_in = node, c_out
    _link(layers, edges)
    return layers, edges


def resnet32_layers(N: int = 128, image: int = 32) -> Tuple[List[ConvSpec], List[Edge]]:
    """The 33 convolutions of a CIFAR ResNet-32 with 1x1 stride-2 projections."""
    layers: List[ConvSpec] = []
    edges: List[Edge] = []

    def new_edge(name: str, n: int) -> int:
        edges.append(Edge(name, n))
        return len(edges) - 1

    h = image
    node = new_edge("stage1_node", 16)
    layers.append(ConvSpec("stem", N, h, h, 3, 16, 3, 3, 1, 1, None, node, first=True))
    c_in = 16
    for si, width in enumerate([16, 32, 64]):
        stage = si + 1
        if stage > 1:
            prev, node = node, new_edge(f"stage{stage}_node", width)
        for b in range(5):
            st = 2 if (b == 0 and stage > 1) else 1
            src, c_src = (prev, c_in) if (b == 0 and stage > 1) else (node, width)
            e = new_edge(f"stage{stage}_b{b}", width)
            layers.append(ConvSpec(f"stage{stage}_b{b}_a", N, h, h, c_src, width, 3, 3, st, 1, src, e))
            ho = h // st
            layers.append(ConvSpec(f"stage{stage}_b{b}_b", N, ho, ho, width, width, 3, 3, 1, 1, e, node))
            if b == 0 and stage > 1:
                layers.append(ConvSpec(f"stage{stage}_proj", N, h, h, c_src, width, 1, 1, 2, 0, src, node))
            h = ho
        c_in = width
    _link(layers, edges)
    return layers, edges


def distinct_shapes(layers: List[ConvSpec]) -> List[Tuple[ConvSpec, int]]:
    """Unique layer shapes in first-appearance order with their multiplicity."""
    seen: Dict[Tuple[int, ...], List] = {}
    for l in layers:
        k = l.shape_key() + (l.first,)
        if k in seen:
            seen[k][1] += 1
        else:
            seen[k] = [l, 1]
    return [(v[0], v[1]) for v in seen.values()]


# --------------------------------------------------------------------------- #
# pruned (ragged) widths and zero patterns
# --------------------------------------------------------------------------- #
def pruned_keep_sets(edges: List[Edge], seed: int = 3, lo: float = 0.4, hi: float = 0.9) -> List[np.ndarray]:
    """Per edge: sorted surviving channel ids.  Keep fraction ~ U[lo, hi]; a count
    that would be a multiple of 16 is lowered by one so every width is ragged."""
    rng = np.random.Generator(np.random.PCG64(seed))
    keep = []
    for e in edges:
        f = rng.uniform(lo, hi)
        n2 = max(1, int(round(f * e.n)))
        if n2 % 16 == 0:
            n2 -= 1
        n2 = max(1, n2)
        keep.append(np.sort(rng.permutation(e.n)[:n2]).astype(np.int32))
    return keep


def with_widths(layers: List[ConvSpec], edges: List[Edge], widths: List[int]) -> Tuple[List[ConvSpec], List[Edge]]:
    """The same network built already compacted: edge e has widths[e] channels."""
    new_layers = [
        replace(
            l,
            C=l.C if l.in_edge is None else widths[l.in_edge],
            K=l.K if l.out_edge is None else widths[l.out_edge],
        )
        for l in layers
    ]
    new_edges = [Edge(e.name, widths[i]) for i, e in enumerate(edges)]
    _link(new_layers, new_edges)
    return new_layers, new_edges


def zeroed_channel_sets(edges: List[Edge], frac: float, rng: np.random.Generator) -> List[np.ndarray]:
    """Per edge: round(frac*n) distinct channel ids to be zeroed (sorted)."""
    out = []
    for e in edges:
        nz = int(round(frac * e.n))
        nz = min(nz, e.n - 1)
        out.append(np.sort(rng.choice(e.n, nz, replace=False)).astype(np.int32))
    return out


# --------------------------------------------------------------------------- #
# tensors
# --------------------------------------------------------------------------- #
def he_std(spec: ConvSpec) -> float:
    return float(np.sqrt(2.0 / (spec.R * spec.S * spec.C)))


def conv_tensors(spec: ConvSpec, rng: np.random.Generator, want=("x", "w", "dy")) -> Dict[str, np.ndarray]:
    """x ~ N(0,1) [N,H,W,C], w ~ He-normal [K,R,S,C], dy ~ N(0,1) [N,P,Q,K], drawn in
    that order as fp32 and rounded to the bf16 grid (still stored as fp32)."""
    out: Dict[str, np.ndarray] = {}
    if "x" in want:
        out["x"] = to_bf16_grid(rng.standard_normal((spec.N, spec.H, spec.W, spec.C), dtype=np.float32))
    if "w" in want:
        w = rng.standard_normal((spec.K, spec.R, spec.S, spec.C), dtype=np.float32) * np.float32(he_std(spec))
        out["w"] = to_bf16_grid(w)
    if "dy" in want:
        out["dy"] = to_bf16_grid(rng.standard_normal((spec.N, spec.P, spec.Q, spec.K), dtype=np.float32))
    return out


def master_weights(spec: ConvSpec, rng: np.random.Generator) -> np.ndarray:
    """fp32 master weights (not rounded): He-normal [K,R,S,C]."""
    return rng.standard_normal((spec.K, spec.R, spec.S, spec.C), dtype=np.float32) * np.float32(he_std(spec))


def zero_groups_in_weights(w: np.ndarray, out_ids, in_ids) -> np.ndarray:
    """Set whole output filters and whole input-channel slices to exact zero."""
    w = w.copy()
    if out_ids is not None and len(out_ids):
        w[np.asarray(out_ids), :, :, :] = 0.0
    if in_ids is not None and len(in_ids):
        w[:, :, :, np.asarray(in_ids)] = 0.0
    return w


def network_weights(layers: List[ConvSpec], edges: List[Edge], zero_sets: Optional[List[np.ndarray]],
                    rng: np.random.Generator, bf16: bool = False) -> List[np.ndarray]:
    """Master weights of every layer, with the edges' zeroed channels written as exact
    zeros in all producers' output groups and all consumers' input groups."""
    ws = []
    for l in layers:
        w = master_weights(l, rng)
        if bf16:
            w = to_bf16_grid(w)
        if zero_sets is not None:
            oz = zero_sets[l.out_edge] if l.out_edge is not None else None
            iz = zero_sets[l.in_edge] if l.in_edge is not None else None
            w = zero_groups_in_weights(w, oz, iz)
        ws.append(w)
    return ws


def cfg1(seed: int = 0) -> Dict[str, object]:
    """Single 3x3 layer, N=4, C=K=16, 16x16, stride 1, pad 1; four output and four
    input channel groups exactly zero; lambda 1e-3, threshold 1e-6."""
    rng = np.random.Generator(np.random.PCG64(seed))
    spec = ConvSpec("cfg1", 4, 16, 16, 16, 16, 3, 3, 1, 1, None, None)
    x = rng.standard_normal((4, 16, 16, 16), dtype=np.float32)
    w = rng.standard_normal((16, 3, 3, 16), dtype=np.float32) * np.float32(0.1)
    zo = np.sort(rng.choice(16, 4, replace=False))
    zi = np.sort(rng.choice(16, 4, replace=False))
    w = zero_groups_in_weights(w, zo, zi)
    dy = rng.standard_normal((4, 16, 16, 16), dtype=np.float32)
    return dict(spec=spec, x=to_bf16_grid(x), w_master=w, w=to_bf16_grid(w), dy=to_bf16_grid(dy),
                zero_out=zo, zero_in=zi, lam=1e-3, thr=1e-6)


def sample_indices(total: int, n: int, rng: np.random.Generator) -> np.ndarray:
    """n distinct flat indices in [0,total), sorted (all of them if n >= total)."""
    if n >= total:
        return np.arange(total, dtype=np.int64)
    return np.sort(rng.choice(total, n, replace=False)).astype(np.int64)
