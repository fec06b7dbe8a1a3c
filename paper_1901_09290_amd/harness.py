"""Device-side harness: per-layer buffers in the layout the library consumes, and the call
sequences of one training step (Alg. 1 lines ForwardProp .. BackProp, per conv layer) and of one
reconfiguration sweep (PruneAndReconfigNetwork).  torch allocates and fills memory; every
computation is a call into the C-ABI library through `binding`.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from . import workloads as wl

DEV = "cuda:0"
# Side streams the weight gradients alternate between.  Measured on the ResNet-50 step: 1 stream 227, 2 streams 239,
# 4 streams 245 TFLOP/s (8 the same; odd counts fall back to ~230, the caller's stream then shares a hardware queue
# with a busy side stream).
WGRAD_STREAMS = 4
# Group norms of this many leading layers precede the forward pass; the rest run beside its first convolutions.  With the
# whole network's norms at ~45 us the split no longer pays (11 leading layers: 7.165 ms per step, all layers: 7.125 ms),
# so by default every layer is a leading one; the k-innermost weight copies still run beside the forward pass.
NORMS_HEAD_LAYERS = 1 << 30


def pitch8(n: int) -> int:
    """Channel pitch used for every tensor: the next multiple of 8 elements (16 bytes of bf16)."""
    return (n + 7) // 8 * 8


def _to_dev_bf16(a: np.ndarray, pitch: int) -> torch.Tensor:
    bits = wl.bf16_bits(a)
    if pitch != a.shape[-1]:
        full = np.zeros(a.shape[:-1] + (pitch,), dtype=np.uint16)
        full[..., : a.shape[-1]] = bits
        bits = full
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def _to_dev_f32(a: np.ndarray, pitch: int) -> torch.Tensor:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if pitch != a.shape[-1]:
        full = np.zeros(a.shape[:-1] + (pitch,), dtype=np.float32)
        full[..., : a.shape[-1]] = a
        a = full
    return torch.from_numpy(a).to(DEV)


class ConvLayer:
    """All device buffers of one convolution layer's training step."""

    def __init__(self, spec: wl.ConvSpec, gen: Optional[torch.Generator] = None,
                 host: Optional[Dict[str, np.ndarray]] = None, w_master: Optional[np.ndarray] = None):
        s = self.spec = spec
        self.xp, self.yp, self.wp = pitch8(s.C), pitch8(s.K), pitch8(s.C)
        # every buffer below starts zeroed and no library call writes padding channels: the padding stays zero
        self.desc = B.desc_of(s, self.xp, self.yp, self.wp, B.CONV_PAD_ZERO)
        self.RS = s.R * s.S
        bf, f32 = torch.bfloat16, torch.float32
        if host is not None:
            self.x = _to_dev_bf16(host["x"], self.xp)
            self.dy = _to_dev_bf16(host["dy"], self.yp)
            wm = host["w"] if w_master is None else w_master
            self.w_master = _to_dev_f32(wm, self.wp)
        else:
            assert gen is not None
            self.x = torch.zeros((s.N, s.H, s.W, self.xp), dtype=bf, device=DEV)
            self.x[..., : s.C].normal_(generator=gen)
            self.dy = torch.zeros((s.N, s.P, s.Q, self.yp), dtype=bf, device=DEV)
            self.dy[..., : s.K].normal_(generator=gen)
            self.w_master = torch.zeros((s.K, s.R, s.S, self.wp), dtype=f32, device=DEV)
            if w_master is not None:
                self.w_master[..., : s.C] = torch.from_numpy(np.ascontiguousarray(w_master, dtype=np.float32)).to(DEV)
            else:
                self.w_master[..., : s.C].normal_(std=wl.he_std(s), generator=gen)
        self.w_bf16 = torch.zeros((s.K, s.R, s.S, self.wp), dtype=bf, device=DEV)
        # the same weights with k innermost, for the input-gradient GEMM (refreshed once per iteration)
        self.w_crsk = None if s.first else torch.zeros((s.C, s.R, s.S, self.yp), dtype=bf, device=DEV)
        self.y = torch.zeros((s.N, s.P, s.Q, self.yp), dtype=bf, device=DEV)
        self.dx = None if s.first else torch.zeros((s.N, s.H, s.W, self.xp), dtype=bf, device=DEV)
        self.dw = torch.zeros((s.K, s.R, s.S, self.wp), dtype=f32, device=DEV)
        self.out_norm = torch.zeros(s.K, dtype=f32, device=DEV)
        self.in_norm = torch.zeros(s.C, dtype=f32, device=DEV)
        self.lasso_flags = B.LASSO_OUT | (0 if s.first else B.LASSO_IN)

    def workspace_bytes(self) -> int:
        d = self.desc
        return max(B.conv_fwd_workspace_bytes(d), B.conv_bwd_data_workspace_bytes(d),
                   B.conv_bwd_weight_workspace_bytes(d), B.conv_bwd_weight_lasso_workspace_bytes(d),
                   B.group_norms_workspace_bytes(self.spec.K, self.RS, self.spec.C))

    def norms_job(self, shadow: bool = True) -> B.LayerWeights:
        s = self.spec
        return B.layer_weights(self.w_master, s.K, self.RS, s.C, self.wp, self.out_norm, self.in_norm,
                               self.w_bf16 if shadow else None)

    def lasso_job(self) -> B.LayerLasso:
        s = self.spec
        return B.layer_lasso(self.w_master, self.out_norm, self.in_norm, self.dw, s.K, self.RS, s.C, self.wp,
                             self.lasso_flags)

    # --- the five calls of one training step on this layer, in Alg. 1 order -------------------- #
    def norms(self, ws, shadow: bool = True):
        s = self.spec
        B.group_norms(self.w_master, s.K, self.RS, s.C, self.wp, self.out_norm, self.in_norm,
                      self.w_bf16 if shadow else None, ws)

    def fwd(self, ws):
        B.conv_fwd(self.desc, self.x, self.w_bf16, self.y, ws)

    def bwd_data(self, ws):
        if self.dx is not None:
            B.conv_bwd_data(self.desc, self.dy, self.w_bf16, self.dx, ws)

    def bwd_data_crsk(self):
        if self.dx is not None:
            B.conv_bwd_data_crsk(self.desc, self.dy, self.w_crsk, self.dx)

    def bwd_weight(self, ws):
        B.conv_bwd_weight(self.desc, self.x, self.dy, self.dw, ws)

    def bwd_weight_lasso(self, ws, lam: float):
        """Weight gradient with the regulariser's gradient added in its reduction pass (dw written once)."""
        B.conv_bwd_weight_lasso(self.desc, self.x, self.dy, self.w_master, self.out_norm, self.in_norm, lam,
                                self.lasso_flags, self.dw, ws)

    def lasso(self, lam: float):
        s = self.spec
        B.group_lasso_grad(self.w_master, self.out_norm, self.in_norm, lam, self.lasso_flags, self.dw, s.K, self.RS,
                           s.C, self.wp)

    def train_step(self, ws, lam: float):
        self.norms(ws)
        self.fwd(ws)
        self.bwd_data(ws)
        self.bwd_weight(ws)
        self.lasso(lam)

    @property
    def step_flops(self) -> int:
        return self.spec.flops * (2 if self.spec.first else 3)


def make_workspace(layers: Sequence[ConvLayer]) -> torch.Tensor:
    n = max([l.workspace_bytes() for l in layers] + [256])
    return torch.empty(n, dtype=torch.uint8, device=DEV)


def build_network(specs: Sequence[wl.ConvSpec], seed: int) -> List[ConvLayer]:
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    return [ConvLayer(s, gen=gen) for s in specs]


class Network:
    """A list of conv layers plus the prepared multi-layer descriptor tables and workspaces."""

    def __init__(self, layers: Sequence[ConvLayer]):
        self.layers = list(layers)
        self.norm_jobs = (B.LayerWeights * len(self.layers))(*[l.norms_job() for l in self.layers])
        # the same jobs in two batches: the forward pass may start once the first layers' bf16 weights exist
        nj = [l.norms_job() for l in self.layers]
        self.norm_head = min(NORMS_HEAD_LAYERS, len(nj))
        self.norm_jobs_head = (B.LayerWeights * self.norm_head)(*nj[: self.norm_head])
        self.norm_jobs_tail = (B.LayerWeights * (len(nj) - self.norm_head))(*nj[self.norm_head:]) if len(nj) > self.norm_head else None
        self.lasso_jobs = (B.LayerLasso * len(self.layers))(*[l.lasso_job() for l in self.layers])
        self.ws_norms = torch.empty(max(256, B.group_norms_batched_workspace_bytes(self.norm_jobs)), dtype=torch.uint8,
                                    device=DEV)
        self.ws = make_workspace(self.layers)
        self.ws_norms_tail = torch.empty_like(self.ws_norms)
        crsk = [B.layer_crsk(l.w_bf16, l.w_crsk, l.spec.K, l.RS, l.spec.C, l.wp) for l in self.layers
                if l.w_crsk is not None]
        self.crsk_jobs = (B.LayerCrsk * len(crsk))(*crsk) if crsk else None
        pen = [B.layer_penalty(l.out_norm, l.in_norm, l.spec.K, l.spec.C, l.lasso_flags) for l in self.layers]
        self.penalty_jobs = (B.LayerPenalty * len(pen))(*pen)
        self.penalty = torch.zeros(1, dtype=torch.float64, device=DEV)
        # Shortcut branches: layer i is one when it reads the same edge as an earlier layer j, the layers j .. i-1 are a
        # chain (each reads what the one before writes) and i writes the edge the chain ends on.  fork[j] = i, and the
        # branch joins the chain after layer i - 1 (forward) / after layer j (backward).
        self.fork: Dict[int, int] = {}
        for i, l in enumerate(self.layers):
            si = l.spec
            if si.in_edge is None or i == 0 or self.layers[i - 1].spec.out_edge != si.out_edge:
                continue
            j = i - 1
            while j > 0 and self.layers[j].spec.in_edge == self.layers[j - 1].spec.out_edge and self.layers[j].spec.in_edge != si.in_edge:
                j -= 1
            if j < i and self.layers[j].spec.in_edge == si.in_edge and j not in self.fork:
                self.fork[j] = i
        self.branch_of = {i: j for j, i in self.fork.items()}
        # The input gradient of a shortcut convolution leaves the input-gradient chain: it starts from the same dy as
        # the residual branch's and is needed only where the block's input gradient is put together, so it runs behind
        # the shortcut's weight gradient on that one's side stream (train step -0.8 %).  On a stream of its own - a
        # sixth stream on four hardware queues - the step gets 11 % slower; the shortcut's forward convolution beside
        # the residual branch's changes nothing measurable and stays in line.
        self.overlap_branches = True
        # In the forward pass the shortcut convolution and the first convolution of the residual branch (same input,
        # independent outputs) go out in one call: where both take the same instantiation of the direct kernel they
        # share a launch, with no stream of their own and no cross-stream dependency.
        self.batch_branches_fwd = True
        self.fwd_pairs = {j: B.conv_fwd_jobs([self.layers[k].desc for k in (j, i)], [self.layers[k].x for k in (j, i)],
                                             [self.layers[k].w_bf16 for k in (j, i)], [self.layers[k].y for k in (j, i)])
                          for j, i in self.fork.items()}
        # weight gradients run on a second stream, off the critical path of the input-gradient chain
        self.sides = [torch.cuda.Stream() for _ in range(WGRAD_STREAMS)]
        self.ws_sides = [self.ws] + [torch.empty_like(self.ws) for _ in range(WGRAD_STREAMS - 1)]
        self.overlap_wgrad = True
        self.fuse_lasso = True   # regulariser's gradient inside the weight gradient's reduction pass

    def train_step(self, lam: float) -> None:
        """Alg. 1, one iteration restricted to the conv layers: GroupLassoReg (all layers' group norms, which
        also refreshes the bf16 weights the convolutions read), ForwardProp, BackProp (input and weight
        gradients, last layer first), then the regulariser's gradient added onto every dW.

        BackProp has two-way parallelism in any network: layer l's weight gradient needs only dy(l), which the
        input gradient of layer l+1 produces, and nothing downstream waits for it.  So the input-gradient chain
        stays on the caller's stream and each weight gradient is enqueued on a side stream behind the event that
        marks its dy as ready.  Weight gradients of different layers are independent of each other as well, so
        they alternate between WGRAD_STREAMS side streams (each with its own split workspace): one layer's short
        reduction pass and the ramp-down of its main kernel overlap the next layer's main kernel.  In this mode the
        regulariser's gradient is added by each weight gradient's own reduction pass (fuse_lasso), so dW is written
        once and no pass over all weights follows the join."""
        if not self.overlap_wgrad:
            B.group_norms_batched(self.norm_jobs, self.ws_norms)
            if self.crsk_jobs is not None:
                B.weights_to_crsk_batched(self.crsk_jobs)
            for l in self.layers:
                l.fwd(self.ws)
        else:
            # The forward pass needs layer l's bf16 weights only when it reaches layer l, and the k-innermost copies
            # only in the backward pass: the first layers' norms run on the caller's stream, the remaining norms and
            # the copies beside the first forward convolutions.
            main, side = torch.cuda.current_stream(), self.sides[0]
            side.wait_stream(main)
            B.group_norms_batched(self.norm_jobs_head, self.ws_norms)
            head_ready = torch.cuda.Event()
            head_ready.record(main)
            with torch.cuda.stream(side):
                if self.norm_jobs_tail is not None:
                    B.group_norms_batched(self.norm_jobs_tail, self.ws_norms_tail)
                tail_ready = torch.cuda.Event()
                tail_ready.record(side)
                if self.crsk_jobs is not None:
                    side.wait_event(head_ready)    # the copies read every layer's bf16 weights, the head layers' too
                    B.weights_to_crsk_batched(self.crsk_jobs)
            pairs = self.batch_branches_fwd and all(i < self.norm_head for i in self.branch_of)
            for i, l in enumerate(self.layers):
                if i == self.norm_head:
                    main.wait_event(tail_ready)
                if pairs and i in self.fork:
                    B.conv_fwd_batched(self.fwd_pairs[i])
                elif not (pairs and i in self.branch_of):
                    l.fwd(self.ws)
            main.wait_stream(side)                 # the k-innermost weight copies are final
        if not self.overlap_wgrad:
            for l in reversed(self.layers):
                l.bwd_data_crsk()
                l.bwd_weight(self.ws)
        else:
            main = torch.cuda.current_stream()
            n = len(self.layers)
            pending: Dict[int, torch.cuda.Event] = {}
            for i, l in enumerate(reversed(self.layers)):
                li = n - 1 - i
                side, ws = self.sides[i % len(self.sides)], self.ws_sides[i % len(self.sides)]
                ready = torch.cuda.Event()
                ready.record(main)                 # dy(l) is final here (the layer above has produced it)
                side.wait_event(ready)
                with torch.cuda.stream(side):      # each workspace is used by one stream only
                    if self.fuse_lasso:
                        l.bwd_weight_lasso(ws, lam)
                    else:
                        l.bwd_weight(ws)
                if self.overlap_branches and li in self.branch_of:
                    with torch.cuda.stream(side):  # behind this layer's weight gradient on the same side stream
                        l.bwd_data_crsk()
                    joined = torch.cuda.Event()
                    joined.record(side)
                    pending[self.branch_of[li]] = joined
                else:
                    l.bwd_data_crsk()
                if li in pending:
                    main.wait_event(pending.pop(li))   # the block's input gradient is complete
            for side in self.sides:
                main.wait_stream(side)
            if self.fuse_lasso:
                return
        B.group_lasso_grad_batched(self.lasso_jobs, lam)

    def regulariser_value(self) -> None:
        """GroupLassoReg of Alg. 1 from the norms of the last train_step / norms call: one launch, result in
        self.penalty (device fp64 scalar).  With the first iteration's classification loss it gives the
        coefficient through binding.lasso_set_coeff (SetCoeff)."""
        B.group_lasso_penalty_batched(self.penalty_jobs, self.penalty)

    def optimizer_step(self, lam: float, lr: float, momentum: float, weight_decay: float) -> None:
        """Optimizer of Alg. 1 with the regulariser's gradient folded in: one pass over w, dw and the momentum
        buffers of all layers (instead of group_lasso_grad_batched followed by an update pass)."""
        if not hasattr(self, "update_jobs"):
            self.mom = [torch.zeros_like(l.w_master) for l in self.layers]
            jobs = [B.layer_update(l.w_master, l.dw, m, l.out_norm, l.in_norm, l.spec.K, l.RS, l.spec.C, l.wp,
                                   l.lasso_flags) for l, m in zip(self.layers, self.mom)]
            self.update_jobs = (B.LayerUpdate * len(jobs))(*jobs)
        B.sgd_momentum_lasso_batched(self.update_jobs, lam, lr, momentum, weight_decay)

    def _bn_state(self):
        if not hasattr(self, "bn"):
            C = max(l.spec.K for l in self.layers)
            elems = max(l.y.numel() for l in self.layers)
            pix = max(l.spec.N * l.spec.P * l.spec.Q for l in self.layers)
            self.bn = {
                "out": torch.empty(elems, dtype=torch.bfloat16, device=DEV),
                "gamma": torch.ones(C, device=DEV), "beta": torch.zeros(C, device=DEV),
                "stat": [torch.empty((2, l.spec.K), device=DEV) for l in self.layers],
                "grad": torch.empty((2, C), device=DEV),
                "ws": torch.empty(max(B.bn_workspace_bytes(l.spec.N * l.spec.P * l.spec.Q, l.spec.K)
                                      for l in self.layers), dtype=torch.uint8, device=DEV),
            }
        return self.bn

    def bn_fwd_all(self, eps: float = 1e-5) -> None:
        """Feature normalisation (training mode) of every convolution's output, layer by layer."""
        st = self._bn_state()
        for l, ms in zip(self.layers, st["stat"]):
            s = l.spec
            B.bn_fwd(l.y, s.N * s.P * s.Q, s.K, l.yp, st["gamma"], st["beta"], eps, st["out"], l.yp, ms[0], ms[1], st["ws"])

    def bn_bwd_all(self) -> None:
        """Its backward pass with each layer's dy as the upstream gradient (after bn_fwd_all)."""
        st = self._bn_state()
        for l, ms in zip(self.layers, st["stat"]):
            s = l.spec
            B.bn_bwd(l.y, l.dy, s.N * s.P * s.Q, s.K, l.yp, l.yp, st["gamma"], ms[0], ms[1], st["out"], l.yp,
                     st["grad"][0], st["grad"][1], st["ws"])

    def fwd_bn_all(self, fused: bool, eps: float = 1e-5) -> None:
        """Every layer's forward convolution followed by the normalisation of its output: as two separate calls
        (three passes over the activation), or with the statistics reduced in the convolution's epilogue (two)."""
        st = self._bn_state()
        if "sums" not in st:
            sizes = [B.conv_fwd_stats_workspace(l.desc) for l in self.layers]
            st["sums"] = torch.empty(max(n for n, _ in sizes), dtype=torch.uint8, device=DEV)
            st["n_partial"] = [k for _, k in sizes]
        for l, ms, npart in zip(self.layers, st["stat"], st["n_partial"]):
            s = l.spec
            pixels = s.N * s.P * s.Q
            if fused:
                B.conv_fwd_stats(l.desc, l.x, l.w_bf16, l.y, st["sums"])
                B.bn_fwd_from_sums(l.y, pixels, s.K, l.yp, st["sums"], npart, st["gamma"], st["beta"], eps, st["out"], l.yp,
                                   ms[0], ms[1])
            else:
                l.fwd(self.ws)
                B.bn_fwd(l.y, pixels, s.K, l.yp, st["gamma"], st["beta"], eps, st["out"], l.yp, ms[0], ms[1], st["ws"])

    @property
    def bn_elements(self) -> int:
        return sum(l.spec.N * l.spec.P * l.spec.Q * l.spec.K for l in self.layers)

    @property
    def step_flops(self) -> int:
        return sum(l.step_flops for l in self.layers)


def train_step(layers: Sequence[ConvLayer], ws: torch.Tensor, lam: float) -> None:
    for l in layers:
        l.train_step(ws, lam)


# ----------------------------------------------------------------------------------------------- #
# reconfiguration sweep
# ----------------------------------------------------------------------------------------------- #
class ReconfigModel:
    """Weights (+ momentum), per-channel normalisation vectors and one saved input activation per
    layer, plus everything the sweep writes: masks, keep masks, index lists and compacted copies."""

    def __init__(self, specs: Sequence[wl.ConvSpec], edges: Sequence[wl.Edge], weights: Sequence[np.ndarray],
                 seed: int, with_activations: bool = True):
        self.specs, self.edges = list(specs), list(edges)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(seed)
        f32, bf, u8, i32 = torch.float32, torch.bfloat16, torch.uint8, torch.int32
        self.w, self.mom, self.bn, self.act = [], [], [], []
        self.on, self.inn, self.zo, self.zi = [], [], [], []
        for s, w in zip(self.specs, weights):
            wp = pitch8(s.C)
            self.w.append(_to_dev_f32(w, wp))
            m = torch.zeros_like(self.w[-1])
            m[..., : s.C].normal_(generator=gen)
            self.mom.append(m)
            self.bn.append([torch.randn(s.K, generator=gen, device=DEV, dtype=f32) for _ in range(4)])
            if with_activations:
                a = torch.zeros((s.N, s.H, s.W, pitch8(s.C)), dtype=bf, device=DEV)
                a[..., : s.C].normal_(generator=gen)
                self.act.append(a)
            self.on.append(torch.zeros(s.K, dtype=f32, device=DEV))
            self.inn.append(torch.zeros(s.C, dtype=f32, device=DEV))
            self.zo.append(torch.zeros(s.K, dtype=u8, device=DEV))
            self.zi.append(torch.zeros(s.C, dtype=u8, device=DEV))
        self.keep = [torch.zeros(e.n, dtype=u8, device=DEV) for e in self.edges]
        self.idx = [torch.zeros(e.n, dtype=i32, device=DEV) for e in self.edges]
        self.counts = torch.zeros(len(self.edges), dtype=i32, device=DEV)
        self.norm_jobs = (B.LayerWeights * len(self.specs))(*[
            B.layer_weights(self.w[i], s.K, s.R * s.S, s.C, pitch8(s.C), self.on[i], self.inn[i], None)
            for i, s in enumerate(self.specs)])
        self.ws = torch.empty(max(256, B.group_norms_batched_workspace_bytes(self.norm_jobs)), dtype=torch.uint8,
                              device=DEV)
        self.detect_jobs = (B.LayerDetect * len(self.specs))(*[
            B.layer_detect(self.w[i], s.K, s.R * s.S, s.C, pitch8(s.C), self.on[i], self.inn[i], self.zo[i], self.zi[i])
            for i, s in enumerate(self.specs)])
        # outputs sized for "nothing pruned"; the sweep writes the compacted tensors at their own pitch
        self.w_out = [torch.zeros_like(t) for t in self.w]
        self.mom_out = [torch.zeros_like(t) for t in self.mom]
        self.bn_out = [[torch.zeros_like(v) for v in vs] for vs in self.bn]
        self.act_out = [torch.zeros_like(t) for t in self.act]
        self.new_counts: Optional[np.ndarray] = None
        self.side = torch.cuda.Stream()   # compaction of the small tensors beside the activation gather
        # whole-network job tables of the multi-job calls (built once; they hold device pointers only)
        mask_jobs = []
        for i, s in enumerate(self.specs):
            mask_jobs += [B.norm_mask(self.on[i], s.K, self.zo[i]), B.norm_mask(self.inn[i], s.C, self.zi[i])]
        self.mask_jobs = (B.NormMask * len(mask_jobs))(*mask_jobs)
        self._edge_structs = [B.edge_plan([self.zo[i] for i in e.producers], [self.zi[i] for i in e.consumers], e.n,
                                          self.keep[k], self.idx[k], self.counts[k:k + 1])
                              for k, e in enumerate(self.edges)]
        self.edge_jobs = (B.EdgePlan * len(self.edges))(*self._edge_structs)

    def detect(self, thr: float) -> None:
        """Group norms and zero masks of every layer (the masks come out of the norms' finish pass), then keep
        mask + survivor list of every edge: two multi-job calls, all asynchronous."""
        B.group_norms_detect_batched(self.detect_jobs, thr, self.ws)
        B.reconcile_plan_batched(self.edge_jobs)

    def detect_separate(self, thr: float) -> None:
        """The same detection with the zero masks from a call of their own."""
        B.group_norms_batched(self.norm_jobs, self.ws)
        B.zero_groups_batched(self.mask_jobs, thr)
        B.reconcile_plan_batched(self.edge_jobs)

    def detect_per_call(self, thr: float) -> None:
        """The same detection through the single-tensor calls (one launch per layer / edge)."""
        B.group_norms_batched(self.norm_jobs, self.ws)
        for i, s in enumerate(self.specs):
            B.zero_groups(self.on[i], s.K, thr, self.zo[i])
            B.zero_groups(self.inn[i], s.C, thr, self.zi[i])
        for e, edge in enumerate(self.edges):
            B.reconcile_edge([self.zo[i] for i in edge.producers], [self.zi[i] for i in edge.consumers], edge.n,
                             self.keep[e])
            B.compact_plan(self.keep[e], edge.n, self.idx[e], self.counts[e:e + 1])

    def compact_activations(self, cnt: np.ndarray) -> None:
        """Only the saved activations' gather of compact(): one multi-job call."""
        self.compact(cnt, only_activations=True)

    def compact(self, cnt: Optional[np.ndarray] = None, per_call: bool = False, only_activations: bool = False) -> None:
        """Gathers every tensor with the planned index lists.  The survivor counts size the outputs: they
        are read back here (one synchronising copy) unless the caller already holds them.  Weights, momentum
        the per-channel vectors and the saved activations of all layers go through the multi-job calls."""
        if cnt is None:
            cnt = self.counts.cpu().numpy()
        self.new_counts = cnt
        wjobs, vjobs, ajobs = [], [], []
        for i, s in enumerate(self.specs):
            ik = self.idx[s.out_edge] if s.out_edge is not None else None
            ic = self.idx[s.in_edge] if s.in_edge is not None else None
            Kp = int(cnt[s.out_edge]) if s.out_edge is not None else s.K
            Cp = int(cnt[s.in_edge]) if s.in_edge is not None else s.C
            RS, wp, op = s.R * s.S, pitch8(s.C), pitch8(Cp)
            if per_call:
                B.compact_weights(self.w[i], s.K, RS, s.C, wp, ik, Kp, ic, Cp, self.w_out[i], op)
                B.compact_weights(self.mom[i], s.K, RS, s.C, wp, ik, Kp, ic, Cp, self.mom_out[i], op)
            else:
                wjobs.append(B.gather_weights(self.w[i], s.K, RS, s.C, wp, ik, Kp, ic, Cp, self.w_out[i], op))
                wjobs.append(B.gather_weights(self.mom[i], s.K, RS, s.C, wp, ik, Kp, ic, Cp, self.mom_out[i], op))
            if ik is not None:
                for v, o in zip(self.bn[i], self.bn_out[i]):
                    if per_call:
                        B.compact_vector(v, 4, ik, Kp, o)
                    else:
                        vjobs.append(B.gather_vector(v, 4, ik, Kp, o))
            if self.act and ic is not None:
                if per_call:
                    B.compact_nhwc(self.act[i], s.N * s.H * s.W, s.C, wp, ic, Cp, self.act_out[i], op)
                else:
                    ajobs.append(B.gather_nhwc(self.act[i], s.N * s.H * s.W, s.C, wp, ic, Cp, self.act_out[i], op))
        if only_activations:
            assert not per_call
            if ajobs:
                B.compact_nhwc_batched(ajobs)
        elif not per_call:
            # the weight-shaped tensors and the per-channel vectors are a few launch-bound kernels over 64 MB; they run
            # on a side stream beside the activation gather, which keeps the memory system busy for 0.3 ms by itself
            main = torch.cuda.current_stream()
            before = torch.cuda.Event()
            before.record(main)                    # everything the compaction depends on
            if ajobs:
                B.compact_nhwc_batched(ajobs)      # the long kernel first: it is the caller's stream that must not wait
            self.side.wait_event(before)
            with torch.cuda.stream(self.side):
                B.compact_weights_batched(wjobs)
                B.compact_vector_batched(vjobs)
            main.wait_stream(self.side)

    def sweep(self, thr: float) -> None:
        self.detect(thr)
        self.compact()

    def algorithmic_bytes(self) -> Dict[str, int]:
        """Bytes each kernel family must move for the last sweep (survivors read once, written once)."""
        cnt = self.new_counts
        out = dict(group_norms=0, compact_weights=0, compact_nhwc=0, compact_vector=0)
        for s in self.specs:
            Kp = int(cnt[s.out_edge]) if s.out_edge is not None else s.K
            Cp = int(cnt[s.in_edge]) if s.in_edge is not None else s.C
            out["group_norms"] += 4 * s.params
            out["compact_weights"] += 2 * 2 * 4 * Kp * s.R * s.S * Cp          # weights + momentum, read + write
            if s.out_edge is not None:
                out["compact_vector"] += 4 * 2 * 4 * Kp
            if self.act and s.in_edge is not None:
                out["compact_nhwc"] += 2 * 2 * s.N * s.H * s.W * Cp
        return out
