"""Caller-side plumbing for a training step over one GPU's block of timesteps (Section "Gradient
Checkpoint": a block is run forward, keeping its activations, and gradients then travel through it in
the reverse direction).  Like pipeline.py this owns buffers and the order of library calls only:

    forward    t = 1..T:   A_t by dgnn_delta_rebuild (t >= 2), per layer H = X W, Z = relu(A~_t H) -- every
                           Z is kept; then Y = Z x_1 M
    backward   G = G_Y x_1 M^T (dgnn_mproduct_backward), then t = T..1:
                   per layer, last to first:   G_P = dinv * (Z > 0 ? G : 0)      dgnn_relu_backward
                                               G_H = A~_t^T G_P                  dgnn_spmm on the transposed snapshot
                                               dW += X^T G_H                     dgnn_weight_grad
                                               G   = G_H W^T  (if a layer lies below)   dgnn_input_grad
                   A_{t-1} from A_t by dgnn_delta_rebuild with the added and deleted lists exchanged

For a directed workload the transposed snapshots are a second dynamic graph, rebuilt the same way from the
difference lists sorted by (col, row).  Nothing here computes: every step runs in the HIP kernels.
"""
from __future__ import annotations

from typing import List, Optional, Tuple

import torch

from . import binding as B
from .pipeline import BlockInputs, BlockRunner


class _Chain:
    """CSR slots for a series of snapshots walked forwards or backwards by rebuilds: by default two alternating slots
    plus a kept first snapshot; with `slots` given, one slot per timestep, so that every snapshot of the block stays
    resident and nothing has to be rebuilt on the way back."""

    def __init__(self, n, cap, dev, rowptr1, colidx1, with_dinv: bool, slots: Optional[int] = None):
        self.per_step = slots is not None
        count = slots if self.per_step else 3
        self.rowptr = [torch.empty(n + 1, dtype=torch.int32, device=dev) for _ in range(count)]
        self.colidx = [torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(count)]
        self.dinv = [torch.empty(n, dtype=torch.float32, device=dev) if with_dinv else None for _ in range(count)]
        self.load_first(rowptr1, colidx1)

    def load_first(self, rowptr1, colidx1) -> None:
        """The block's first snapshot, which arrives whole, goes into its slot."""
        k = self.slot_of(1)
        self.rowptr[k].copy_(rowptr1)
        self.colidx[k][: colidx1.numel()].copy_(colidx1)
        if self.dinv[k] is not None:
            B.csr_dinv(self.rowptr[k], self.dinv[k])

    def slot_of(self, t: int) -> int:
        if self.per_step:
            return t - 1
        return 2 if t == 1 else t % 2


class BlockTrainer:
    """Forward and backward over one block; gradients of the layer weights (fp32) come out in `dw`."""

    def __init__(self, blk: BlockInputs, directed: bool,
                 transposed_first: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
                 transposed_deltas: Optional[List[Tuple[torch.Tensor, ...]]] = None, want_dx: bool = False,
                 cap: Optional[int] = None, max_list: Optional[int] = None, keep_snapshots: bool = False):
        self.blk = blk
        dev = blk.rowptr1.device
        self.dev = dev
        n, f, T, L = blk.n, blk.f, blk.T, blk.layers
        dt = blk.x[0].dtype
        cap = max(max(blk.nnz), cap or 0)          # room for the densest snapshot this trainer will ever hold
        self.cap, self.T_max = cap, T
        self.t0 = 0                     # timesteps of the series before this block
        self.z_before = None            # last w-1 frames of the top layer's Z before this block
        self.directed = directed
        # keep_snapshots: every A_t (and A_t^T) of the block stays resident (T index arrays instead of three), so the
        # backward pass rebuilds nothing; without, the snapshots are rebuilt in reverse, as gradient checkpointing
        # has it.  4 nnz bytes per snapshot and chain: 9.6 GB for c5's eight, a matter of course in 288 GB.
        self.keep_snapshots = keep_snapshots
        slots = T if keep_snapshots else None
        self.a = _Chain(n, cap, dev, blk.rowptr1, blk.colidx1, with_dinv=True, slots=slots)
        self.at = None
        if directed:
            assert transposed_first is not None and transposed_deltas is not None
            self.at = _Chain(n, cap, dev, transposed_first[0], transposed_first[1], with_dinv=False, slots=slots)
            self.t_deltas = transposed_deltas
        self.z = torch.empty((L, T, n, f), dtype=dt, device=dev)          # activations of the block
        self.y = torch.empty((T, n, f), dtype=dt, device=dev) if blk.window else None
        self.g = None                                                     # dL/dZ of the last layer, if g_y must be kept
        self.h = torch.empty((n, f), dtype=dt, device=dev)                # H going forward, G_H going back
        self.gp = torch.empty((n, f), dtype=dt, device=dev)
        self.g_mid = torch.empty((n, f), dtype=dt, device=dev) if L > 1 else None
        self.dx = torch.empty((T, n, f), dtype=dt, device=dev) if want_dx else None
        self.dw = [torch.zeros((f, f), dtype=torch.float32, device=dev) for _ in range(L)]
        # with one weight per timestep (Section "EvolveGCN") every timestep has a gradient of its own
        self.dw_t = ([[torch.zeros((f, f), dtype=torch.float32, device=dev) for _ in range(L)] for _ in range(T)]
                     if blk.w_t is not None else None)
        max_list = max([int(d[0].numel()) for d in blk.deltas] + [int(d[2].numel()) for d in blk.deltas] + [1, max_list or 0])
        self.ws_rebuild = torch.empty(B.delta_rebuild_workspace(n, cap, max_list, max_list), dtype=torch.uint8, device=dev)
        self.ws_spmm = torch.empty(B.spmm_workspace(n, cap, f), dtype=torch.uint8, device=dev)
        self.ws_wgrad = torch.empty(B.weight_grad_workspace(f, f), dtype=torch.uint8, device=dev)
        self.timer = None

    def rebind(self, blk: BlockInputs, t0: int = 0, z_before: Optional[torch.Tensor] = None,
               transposed_first=None, transposed_deltas=None) -> None:
        """Point the same buffers at another block of the same series (not longer, not denser than the first)."""
        assert blk.T <= self.T_max and max(blk.nnz) <= self.cap and blk.n == self.blk.n and blk.f == self.blk.f
        self.blk, self.t0, self.z_before = blk, t0, z_before
        self.a.load_first(blk.rowptr1, blk.colidx1)
        if self.directed:
            self.at.load_first(*transposed_first)
            self.t_deltas = transposed_deltas

    def _stage(self, name):
        import contextlib
        return self.timer.stage(name) if self.timer is not None else contextlib.nullcontext()

    def _rebuild(self, chain: _Chain, lists, nnz_src: int, src_t: int, dst_t: int, reverse: bool) -> None:
        ar, ac, dr, dc = lists
        if reverse:
            ar, ac, dr, dc = dr, dc, ar, ac
        s, d = chain.slot_of(src_t), chain.slot_of(dst_t)
        with self._stage("delta_rebuild"):
            B.delta_rebuild(chain.rowptr[s], chain.colidx[s], nnz_src, ar, ac, int(ar.numel()), dr, dc, int(dr.numel()),
                            chain.rowptr[d], chain.colidx[d], chain.dinv[d], self.ws_rebuild)

    # ------------------------------------------------------------------ forward, keeping activations
    def forward(self) -> torch.Tensor:
        blk = self.blk
        for t in range(1, blk.T + 1):
            if t >= 2:
                self._rebuild(self.a, blk.deltas[t - 2], blk.nnz[t - 2], t - 1, t, reverse=False)
                if self.directed:
                    self._rebuild(self.at, self.t_deltas[t - 2], blk.nnz[t - 2], t - 1, t, reverse=False)
            slot = self.a.slot_of(t)
            cur = blk.x[t - 1]
            for layer in range(blk.layers):
                with self._stage("feature_transform"):
                    B.feature_transform(cur, blk.weight(t, layer), self.h, row_scale=self.a.dinv[slot])
                with self._stage("spmm"):
                    B.spmm(self.a.rowptr[slot], self.a.colidx[slot], blk.nnz[t - 1], self.a.dinv[slot], self.h,
                           self.z[layer, t - 1], self.ws_spmm, flags=B.DGNN_RELU | B.DGNN_H_PRESCALED)
                cur = self.z[layer, t - 1]
        top = self.z[blk.layers - 1, : blk.T]
        if blk.window:
            with self._stage("mproduct"):
                B.mproduct_block(top, self.y[: blk.T], blk.window, self.t0, z_before=self.z_before)
            return self.y[: blk.T]
        return top

    # ------------------------------------------------------------------ backward
    def backward(self, g_y: torch.Tensor, overwrite: bool = False, g_after: Optional[torch.Tensor] = None,
                 accumulate: bool = False) -> None:
        """g_y [T, n, f] = dL/dY.  Must follow forward() (A_T and, if directed, A_T^T are resident).
        With overwrite the adjoint of the M-transform is taken in place, on g_y itself; g_after = upstream
        gradient of the (up to w-1) timesteps after this block; accumulate adds to dw instead of replacing it."""
        blk = self.blk
        L, T = blk.layers, blk.T
        if blk.window:
            if overwrite:
                g_top = g_y
            else:
                if self.g is None:
                    self.g = torch.empty((self.T_max,) + tuple(g_y.shape[1:]), dtype=g_y.dtype, device=g_y.device)
                g_top = self.g[:T]
            with self._stage("mproduct_backward"):
                B.mproduct_backward_block(g_y, g_top, blk.window, self.t0, g_after=g_after)
        else:
            g_top = g_y
        first_call = [not accumulate] * L
        for t in range(T, 0, -1):
            slot = self.a.slot_of(t)
            tc = self.at if self.directed else self.a           # the chain that holds (A_t + I)^T
            dinv = self.a.dinv[slot]
            g_in = g_top[t - 1]
            for layer in range(L - 1, -1, -1):
                with self._stage("relu_backward"):
                    B.relu_backward(g_in, self.z[layer, t - 1], self.gp, row_scale=dinv)
                with self._stage("spmm_transposed"):
                    B.spmm(tc.rowptr[slot], tc.colidx[slot], blk.nnz[t - 1], dinv, self.gp, self.h, self.ws_spmm,
                           flags=B.DGNN_H_PRESCALED)
                below = blk.x[t - 1] if layer == 0 else self.z[layer - 1, t - 1]
                with self._stage("weight_grad"):
                    if self.dw_t is not None:
                        B.weight_grad(below, self.h, self.dw_t[t - 1][layer], self.ws_wgrad)
                    else:
                        B.weight_grad(below, self.h, self.dw[layer], self.ws_wgrad, accumulate=not first_call[layer])
                first_call[layer] = False
                if layer > 0:
                    with self._stage("input_grad"):
                        B.input_grad(self.h, blk.weight(t, layer), self.g_mid)
                    g_in = self.g_mid
                elif self.dx is not None:
                    with self._stage("input_grad"):
                        B.input_grad(self.h, blk.weight(t, 0), self.dx[t - 1])
            if t >= 3 and not self.keep_snapshots:   # A_{t-1} from A_t: the same rebuild with the two lists exchanged (A_1 was kept)
                self._rebuild(self.a, blk.deltas[t - 2], blk.nnz[t - 1], t, t - 1, reverse=True)
                if self.directed:
                    self._rebuild(self.at, self.t_deltas[t - 2], blk.nnz[t - 1], t, t - 1, reverse=True)


def capture_training_step(tr: "BlockTrainer", g_y: torch.Tensor) -> "torch.cuda.CUDAGraph":
    """One training step (forward keeping activations, then backward for the upstream gradient g_y) recorded as a HIP
    graph: every library call on the way only enqueues kernels, so the step is capturable, and replaying it costs one
    launch instead of one per kernel, which is what bounds small workloads.  The step is run once eagerly first, so
    that one-time host-side set-up inside the library is not part of the recording.  Replays read g_y and the block's
    inputs where they lie and leave the gradients in tr.dw."""
    tr.forward()
    tr.backward(g_y)
    torch.cuda.synchronize(tr.dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tr.forward()
        tr.backward(g_y)
    return graph


def transposed_inputs(blk: BlockInputs):
    """(rowptr, colidx) of A_1^T and the difference lists of the transposed series (dgnn_csr_transpose,
    dgnn_coo_transpose: input formatting, once per block)."""
    n = blk.n
    first = B.csr_transpose(blk.rowptr1, blk.colidx1, blk.nnz[0])
    return first, [B.coo_transpose(n, ar, ac) + B.coo_transpose(n, dr, dc) for ar, ac, dr, dc in blk.deltas]


def make_smoothed_trainer(wl, blk: BlockInputs, life: int) -> "SmoothedTrainer":
    directed = wl.graph != "er"
    if not directed:
        return SmoothedTrainer(blk, life, False)
    first, deltas = transposed_inputs(blk)
    return SmoothedTrainer(blk, life, True, transposed_first=first, transposed_deltas=deltas)


def make_trainer(wl, blk: BlockInputs, want_dx: bool = False, keep_snapshots: bool = False) -> BlockTrainer:
    """Trainer for a block; for a directed workload the transposed first snapshot and lists are prepared here."""
    directed = wl.graph != "er"
    if not directed:
        return BlockTrainer(blk, False, want_dx=want_dx, keep_snapshots=keep_snapshots)
    first, t_deltas = transposed_inputs(blk)
    return BlockTrainer(blk, True, transposed_first=first, transposed_deltas=t_deltas, want_dx=want_dx,
                        keep_snapshots=keep_snapshots)


class CheckpointedTrainer:
    """The paper's gradient checkpointing over a series of T timesteps cut into blocks (Section "Gradient
    Checkpoint"): a forward pass block by block that keeps only what the next block needs (the last w - 1 frames
    of Z; here also each block's first snapshot, which the paper sends whole), then, from the last block to the
    first, a rerun of the block's forward pass followed by its backward pass.  Activations of one block at a
    time are resident."""

    def __init__(self, wl, series: BlockInputs, bsize: int):
        self.series, self.bsize = series, bsize
        self.directed = wl.graph != "er"
        T = series.T
        self.bounds = [(a, min(a + bsize, T)) for a in range(0, T, bsize)]
        dev = series.rowptr1.device
        # first snapshot of every block: block 0 has it, the others are filled in by the forward pass
        self.first = [(series.rowptr1, series.colidx1)] + [
            (torch.empty_like(series.rowptr1), torch.empty(series.nnz[a], dtype=torch.int32, device=dev))
            for a, _ in self.bounds[1:]]
        self.t_first, self.t_deltas = None, None
        if self.directed:
            (rp_t, tc), self.t_deltas = transposed_inputs(series)
            self.t_first = [(rp_t, tc)] + [(torch.empty_like(rp_t), torch.empty(series.nnz[a], dtype=torch.int32, device=dev))
                                           for a, _ in self.bounds[1:]]
        self.pi: List[Optional[torch.Tensor]] = [None] * len(self.bounds)   # frames handed to block b
        longest_list = max([int(d[0].numel()) for d in series.deltas] + [int(d[2].numel()) for d in series.deltas] + [1])
        self.trainer = BlockTrainer(self._block(0), self.directed,       # block 0 is as long as any
                                    transposed_first=self.t_first[0] if self.directed else None,
                                    transposed_deltas=self._t_deltas(*self.bounds[0]),
                                    cap=max(series.nnz), max_list=longest_list)
        self.dw = self.trainer.dw

    def _block(self, b: int) -> BlockInputs:
        s = self.series
        a, e = self.bounds[b]
        nnz = list(s.nnz[a:e])
        blk = BlockInputs(n=s.n, T=e - a, f=s.f, layers=s.layers, window=s.window, rowptr1=self.first[b][0],
                          colidx1=self.first[b][1], deltas=s.deltas[a:e - 1], x=s.x[a:e], w=s.w,
                          w_t=s.w_t[a:e] if s.w_t is not None else None, nnz=nnz)
        return blk

    def _t_deltas(self, a: int, e: int):
        return self.t_deltas[a:e - 1] if self.directed else None

    def _bind(self, b: int) -> None:
        a, e = self.bounds[b]
        self.trainer.rebind(self._block(b), t0=a, z_before=self.pi[b],
                            transposed_first=self.t_first[b] if self.directed else None,
                            transposed_deltas=self._t_deltas(a, e))

    def forward(self, on_block=None) -> None:
        """Block by block; on_block(b, a, e, y) sees the block's output frames before they are overwritten."""
        s, tr = self.series, self.trainer
        w1 = max(s.window - 1, 0)
        for b, (a, e) in enumerate(self.bounds):
            self._bind(b)
            y = tr.forward()
            if on_block is not None:
                on_block(b, a, e, y)
            if b + 1 < len(self.bounds):
                if w1:
                    top = tr.z[s.layers - 1, : e - a]
                    keep = min(w1, e)                       # frames of the series so far that the window reaches
                    own = top[max(e - a - keep, 0):]
                    if own.shape[0] < keep:                 # a block shorter than the window: older frames come along
                        own = torch.cat([self.pi[b][-(keep - own.shape[0]):], own])
                    self.pi[b + 1] = own.clone()
                # the next block's first snapshot (the paper sends it whole; here it is one more rebuild)
                slot = tr.a.slot_of(e - a)
                ar, ac, dr, dc = s.deltas[e - 1]
                B.delta_rebuild(tr.a.rowptr[slot], tr.a.colidx[slot], s.nnz[e - 1], ar, ac, int(ar.numel()), dr, dc,
                                int(dr.numel()), self.first[b + 1][0], self.first[b + 1][1], None, tr.ws_rebuild)
                if self.directed:
                    ar, ac, dr, dc = self.t_deltas[e - 1]
                    B.delta_rebuild(tr.at.rowptr[slot], tr.at.colidx[slot], s.nnz[e - 1], ar, ac, int(ar.numel()), dr,
                                    dc, int(dr.numel()), self.t_first[b + 1][0], self.t_first[b + 1][1], None,
                                    tr.ws_rebuild)

    def backward(self, g_y: torch.Tensor) -> None:
        """g_y [T, n, f] for the whole series.  Must follow forward()."""
        s, tr = self.series, self.trainer
        w1 = max(s.window - 1, 0)
        last = len(self.bounds) - 1
        for b in range(last, -1, -1):
            a, e = self.bounds[b]
            self._bind(b)
            tr.forward()                                                    # the rerun
            after = g_y[e:min(e + w1, s.T)] if (w1 and e < s.T) else None
            tr.backward(g_y[a:e], g_after=after, accumulate=b != last)


class _Ring:
    """`slots` CSR slots used in turn by the raw snapshots A_1, A_2, ...: A_{t-life} is still resident when A_t is."""

    def __init__(self, n, cap, dev, slots: int, with_dinv: bool):
        self.slots = slots
        self.rowptr = [torch.empty(n + 1, dtype=torch.int32, device=dev) for _ in range(slots)]
        self.colidx = [torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(slots)]
        self.dinv = [torch.empty(n, dtype=torch.float32, device=dev) if with_dinv else None for _ in range(slots)]

    def slot_of(self, t: int) -> int:
        return t % self.slots

    def load_first(self, rowptr1, colidx1) -> None:
        s = self.slot_of(1)
        self.rowptr[s].copy_(rowptr1)
        self.colidx[s][: colidx1.numel()].copy_(colidx1)

    def snapshot(self, t: int, nnz: int):
        s = self.slot_of(t)
        return self.rowptr[s], self.colidx[s], nnz


class SmoothedTrainer:
    """A training step on SMOOTHED snapshots (Section "Smoothening the Input Graphs": the graphs TM-GCN and EvolveGCN
    are trained on), with the smoothing done on the device.  Forward: the raw A_t by dgnn_delta_rebuild,
    S_t = S_{t-1} + A_t - A_{t-life} by dgnn_csr_combine, its normalisation by dgnn_csr_weighted_dinv, then per layer
    H = X W and Z = relu(D^(-1/2) S_t D^(-1/2) H) with the counts as values (dgnn_spmm_weighted).  Every S_t stays
    resident (index and value arrays of all T smoothed snapshots: 21 GB at c5's size; and as many again for the
    transposed ones of a directed workload), so the backward pass needs no graph work at all: it is the one of
    BlockTrainer with the weighted aggregation on S_t^T.  Buffers and call order only."""

    def __init__(self, blk: BlockInputs, life: int, directed: bool,
                 transposed_first: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
                 transposed_deltas: Optional[List[Tuple[torch.Tensor, ...]]] = None, diag_value: float = 1.0):
        self.blk, self.life, self.directed = blk, life, directed
        # edge-life smoothing acts on A; Eqn (1) then adds the self loop once: the stored diagonal stays 1 (0.0 here
        # leaves the summed diagonal min(life, t), which is the M-transform of the adjacency tensor instead)
        self.diag_value = diag_value
        dev = blk.rowptr1.device
        self.dev = dev
        n, f, T, L = blk.n, blk.f, blk.T, blk.layers
        dt = blk.x[0].dtype
        cap = max(blk.nnz)
        max_del = max([int(d[2].numel()) for d in blk.deltas] + [0])
        max_list = max([int(d[0].numel()) for d in blk.deltas] + [max_del, 1])
        self.cap_s = cap + life * max_del                  # the window's union: A_t and what the window's steps deleted
        self.raw = _Ring(n, cap, dev, life + 1, with_dinv=False)
        self.raw_t = _Ring(n, cap, dev, life + 1, with_dinv=False) if directed else None
        self.t_first, self.t_deltas = transposed_first, transposed_deltas
        if directed:
            assert transposed_first is not None and transposed_deltas is not None

        def smoothed_slots():
            return [(torch.empty(n + 1, dtype=torch.int32, device=dev), torch.empty(self.cap_s, dtype=torch.int32, device=dev),
                     torch.empty(self.cap_s, dtype=torch.float32, device=dev)) for _ in range(T)]
        self.s = smoothed_slots()
        self.st = smoothed_slots() if directed else self.s
        self.s_nnz = [0] * T
        self.dinv_s = torch.empty((T, n), dtype=torch.float32, device=dev)
        self.z = torch.empty((L, T, n, f), dtype=dt, device=dev)
        self.y = torch.empty((T, n, f), dtype=dt, device=dev) if blk.window else None
        self.g = None
        self.h = torch.empty((n, f), dtype=dt, device=dev)
        self.gp = torch.empty((n, f), dtype=dt, device=dev)
        self.g_mid = torch.empty((n, f), dtype=dt, device=dev) if L > 1 else None
        self.dw = [torch.zeros((f, f), dtype=torch.float32, device=dev) for _ in range(L)]
        # with one weight per timestep (Section "EvolveGCN") every timestep has a gradient of its own
        self.dw_t = ([[torch.zeros((f, f), dtype=torch.float32, device=dev) for _ in range(L)] for _ in range(T)]
                     if blk.w_t is not None else None)
        self.ws_rebuild = torch.empty(B.delta_rebuild_workspace(n, cap, max_list, max_list), dtype=torch.uint8, device=dev)
        self.ws_combine = torch.empty(B.csr_combine_workspace(self.cap_s), dtype=torch.uint8, device=dev)
        self.ws_dinv = torch.empty(B.csr_weighted_dinv_workspace(self.cap_s), dtype=torch.uint8, device=dev)
        self.ws_spmm = torch.empty(B.spmm_workspace(n, self.cap_s, f), dtype=torch.uint8, device=dev)
        self.ws_wgrad = torch.empty(B.weight_grad_workspace(f, f), dtype=torch.uint8, device=dev)
        self.status = torch.zeros(T + 1, dtype=torch.int32, device=dev)     # per timestep: what dgnn_csr_combine found
        self.timer = None

    def _stage(self, name):
        import contextlib
        return self.timer.stage(name) if self.timer is not None else contextlib.nullcontext()

    def _advance(self, ring: _Ring, lists, t: int) -> None:
        ar, ac, dr, dc = lists
        s, d = ring.slot_of(t - 1), ring.slot_of(t)
        with self._stage("delta_rebuild"):
            B.delta_rebuild(ring.rowptr[s], ring.colidx[s], self.blk.nnz[t - 2], ar, ac, int(ar.numel()), dr, dc, int(dr.numel()),
                            ring.rowptr[d], ring.colidx[d], None, self.ws_rebuild)

    def _smooth(self, ring: _Ring, store, t: int) -> None:
        """store[t-1] <- S_t (t >= 2) from store[t-2], A_t and A_{t-life}.  Its number of stored entries stays on the
        device (the last row pointer); the calls that take S_t are given the capacity as an upper bound."""
        blk = self.blk
        prev = store[t - 2] + (self.s_nnz[t - 2],)
        a_out = ring.snapshot(t - self.life, blk.nnz[t - self.life - 1]) if t - self.life >= 1 else None
        with self._stage("csr_combine"):
            B.csr_combine(prev, ring.snapshot(t, blk.nnz[t - 1]), 1.0, a_out, -1.0, store[t - 1], self.ws_combine,
                          diag_value=self.diag_value, status=self.status[t:t + 1])

    def forward(self) -> torch.Tensor:
        blk = self.blk
        self.raw.load_first(blk.rowptr1, blk.colidx1)
        if self.directed:
            self.raw_t.load_first(*self.t_first)
        for t in range(1, blk.T + 1):
            if t == 1:                                  # S_1 = A_1, every entry counted once
                for store, (rp1, ci1) in ((self.s, (blk.rowptr1, blk.colidx1)),) + (((self.st, self.t_first),) if self.directed else ()):
                    store[0][0].copy_(rp1)
                    store[0][1][: blk.nnz[0]].copy_(ci1)
                    store[0][2][: blk.nnz[0]].fill_(1.0)
                self.s_nnz[0] = blk.nnz[0]
            else:
                self._advance(self.raw, blk.deltas[t - 2], t)
                self._smooth(self.raw, self.s, t)
                if self.directed:
                    self._advance(self.raw_t, self.t_deltas[t - 2], t)
                    self._smooth(self.raw_t, self.st, t)
                self.s_nnz[t - 1] = self.cap_s           # an upper bound: the kernels read the count from the last row pointer
            rp, ci, val = self.s[t - 1]
            nnz = self.s_nnz[t - 1]
            with self._stage("csr_weighted_dinv"):
                B.csr_weighted_dinv(rp, val, nnz, self.dinv_s[t - 1], self.ws_dinv)
            cur = blk.x[t - 1]
            for layer in range(blk.layers):
                with self._stage("feature_transform"):
                    B.feature_transform(cur, blk.weight(t, layer), self.h, row_scale=self.dinv_s[t - 1])
                with self._stage("spmm_weighted"):
                    B.spmm_weighted(rp, ci, val, nnz, self.h, self.z[layer, t - 1], self.ws_spmm,
                                    flags=B.DGNN_RELU | B.DGNN_H_PRESCALED, dinv=self.dinv_s[t - 1])
                cur = self.z[layer, t - 1]
        top = self.z[blk.layers - 1]
        if blk.window:
            with self._stage("mproduct"):
                B.mproduct_block(top, self.y, blk.window, 0)
            return self.y
        return top

    def backward(self, g_y: torch.Tensor) -> None:
        """g_y [T, n, f] = dL/dY.  Must follow forward()."""
        blk = self.blk
        L, T = blk.layers, blk.T
        if blk.window:
            if self.g is None:
                self.g = torch.empty_like(g_y)
            with self._stage("mproduct_backward"):
                B.mproduct_backward_block(g_y, self.g, blk.window, 0)
            g_top = self.g
        else:
            g_top = g_y
        first_call = [True] * L
        for t in range(T, 0, -1):
            rp, ci, val = self.st[t - 1]                 # S_t^T (S_t itself for an undirected workload)
            nnz, dinv = self.s_nnz[t - 1], self.dinv_s[t - 1]
            g_in = g_top[t - 1]
            for layer in range(L - 1, -1, -1):
                with self._stage("relu_backward"):
                    B.relu_backward(g_in, self.z[layer, t - 1], self.gp, row_scale=dinv)
                with self._stage("spmm_weighted_transposed"):
                    B.spmm_weighted(rp, ci, val, nnz, self.gp, self.h, self.ws_spmm, flags=B.DGNN_H_PRESCALED, dinv=dinv)
                below = blk.x[t - 1] if layer == 0 else self.z[layer - 1, t - 1]
                with self._stage("weight_grad"):
                    if self.dw_t is not None:
                        B.weight_grad(below, self.h, self.dw_t[t - 1][layer], self.ws_wgrad)
                    else:
                        B.weight_grad(below, self.h, self.dw[layer], self.ws_wgrad, accumulate=not first_call[layer])
                first_call[layer] = False
                if layer > 0:
                    with self._stage("input_grad"):
                        B.input_grad(self.h, blk.weight(t, layer), self.g_mid)
                    g_in = self.g_mid
