"""Caller-side plumbing for one GPU's block of timesteps: owns the device buffers (torch, used
for memory and streams only) and issues the library calls in the order of the forward pass,

    t = 1:      A_1 resident (sent whole, Section "Graph-difference Based Input Transfer")
    t = 2..T:   [difference lists host -> device]  ->  dgnn_delta_rebuild  ->  A_t
    every t:    per GCN layer  H = X W (dgnn_feature_transform),  Z = relu(A~_t H) (dgnn_spmm)
    at the end: Y = Z x_1 M (dgnn_mproduct) when the workload has a window.

No arithmetic of the method lives here; every step runs in the HIP kernels behind the C boundary.
"""
from __future__ import annotations

import contextlib
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

from . import binding as B


@dataclass
class BlockInputs:
    """Inputs of one block of T snapshots, resident on `device`."""
    n: int
    T: int
    f: int
    layers: int
    window: int
    rowptr1: torch.Tensor                  # int32 [n+1]   first snapshot, sent whole
    colidx1: torch.Tensor                  # int32 [nnz_1]
    deltas: List[Tuple[torch.Tensor, ...]]  # per t = 2..T: (add_row, add_col, del_row, del_col), int32, device
    x: List[torch.Tensor]                  # T frames [n, f]
    w: List[torch.Tensor]                  # one weight [f, f] per layer, shared by all timesteps
    w_t: Optional[List[List[torch.Tensor]]] = None   # or one per timestep and layer (Section "EvolveGCN": W_t evolves)
    pinned: Optional[List[Tuple[torch.Tensor, ...]]] = None   # the same lists in pinned host memory
    nnz: List[int] = field(default_factory=list)              # nnz_t, t = 1..T (host arithmetic on list lengths)

    def __post_init__(self):
        if not self.nnz:
            cur = int(self.colidx1.numel())
            self.nnz = [cur]
            for ar, _, dr, _ in self.deltas:
                cur += int(ar.numel()) - int(dr.numel())
                self.nnz.append(cur)

    def weight(self, t: int, layer: int) -> torch.Tensor:
        """The weight of `layer` at timestep t (1-based)."""
        return self.w_t[t - 1][layer] if self.w_t is not None else self.w[layer]


class StageTimer:
    """Per-stage GPU time from event pairs recorded on the stream the kernels are launched on."""

    def __init__(self, device):
        self.device = device
        self.pairs = []          # (stage, start, end)

    @contextlib.contextmanager
    def stage(self, name: str):
        s = torch.cuda.Event(enable_timing=True)
        e = torch.cuda.Event(enable_timing=True)
        stream = torch.cuda.current_stream(self.device)
        s.record(stream)
        try:
            yield
        finally:
            e.record(stream)
            self.pairs.append((name, s, e))

    def totals(self):
        """{stage: (calls, total milliseconds)} -- call after a synchronize."""
        out = {}
        for name, s, e in self.pairs:
            c, ms = out.get(name, (0, 0.0))
            out[name] = (c + 1, ms + s.elapsed_time(e))
        return out


class BlockRunner:
    """Buffers and call sequence for the forward pass over one block."""

    def __init__(self, blk: BlockInputs, keep_all_z: Optional[bool] = None):
        self.blk = blk
        dev = blk.rowptr1.device
        self.dev = dev
        n, f = blk.n, blk.f
        dt = blk.x[0].dtype
        cap = max(blk.nnz)
        self.cap = cap
        # CSR slots: slot 2 keeps A_1 for the whole life of the block (so a pass can be repeated), slots
        # 0 and 1 are used alternately by A_2, A_3, ...: A_{t-1} is read while A_t is written
        self.rowptr = [torch.empty(n + 1, dtype=torch.int32, device=dev) for _ in range(3)]
        self.colidx = [torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(3)]
        self.dinv = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(3)]
        self.h = torch.empty((n, f), dtype=dt, device=dev)
        self.z_mid = torch.empty((n, f), dtype=dt, device=dev) if blk.layers > 1 else None
        self.keep_all_z = bool(blk.window) if keep_all_z is None else keep_all_z
        zt = blk.T if self.keep_all_z else 1
        self.z = torch.empty((zt, n, f), dtype=dt, device=dev)
        max_add = max([int(d[0].numel()) for d in blk.deltas] + [1])
        max_del = max([int(d[2].numel()) for d in blk.deltas] + [1])
        ws_r = B.delta_rebuild_workspace(n, cap, max_add, max_del)
        ws_s = B.spmm_workspace(n, cap, f)
        self.ws_rebuild = torch.empty(ws_r, dtype=torch.uint8, device=dev)
        self.ws_spmm = torch.empty(ws_s, dtype=torch.uint8, device=dev)
        self.status = torch.zeros(blk.T + 1, dtype=torch.int32, device=dev)
        self.timer: Optional[StageTimer] = None
        # staging for difference lists that arrive from pinned host memory (two sets, used alternately)
        self.stage = None
        if blk.pinned is not None:
            self.stage = [tuple(torch.empty(m, dtype=torch.int32, device=dev) for m in (max_add, max_add, max_del, max_del))
                          for _ in range(2)]
            self.copy_stream = torch.cuda.Stream(device=dev)
            self.copied = [torch.cuda.Event() for _ in range(2)]
            self.consumed = [torch.cuda.Event() for _ in range(2)]

    # ------------------------------------------------------------------ pieces
    def _stage(self, name: str):
        return self.timer.stage(name) if self.timer is not None else contextlib.nullcontext()

    @staticmethod
    def slot_of(t: int) -> int:
        return 2 if t == 1 else t % 2

    def load_first(self) -> None:
        """Place A_1 in its slot and derive its dinv (outside any timed region: A_1 is sent whole)."""
        blk = self.blk
        self.rowptr[2].copy_(blk.rowptr1)
        self.colidx[2][: blk.nnz[0]].copy_(blk.colidx1)
        B.csr_dinv(self.rowptr[2], self.dinv[2])

    def rebuild(self, t: int, lists, validate: bool = False) -> None:
        """A_t from A_{t-1} and the difference lists of step t (t >= 2)."""
        blk = self.blk
        src, dst = self.slot_of(t - 1), self.slot_of(t)
        ar, ac, dr, dc = lists
        n_add, n_del = int(blk.deltas[t - 2][0].numel()), int(blk.deltas[t - 2][2].numel())
        with self._stage("delta_rebuild"):
            nnz = B.delta_rebuild(self.rowptr[src], self.colidx[src], blk.nnz[t - 2], ar, ac, n_add, dr, dc, n_del,
                                  self.rowptr[dst], self.colidx[dst], self.dinv[dst], self.ws_rebuild,
                                  flags=B.DGNN_VALIDATE if validate else 0, d_status=self.status[t:t + 1])
        assert nnz == blk.nnz[t - 1]

    def transform_first(self, t: int, h: torch.Tensor) -> None:
        """H = D^(-1/2) (X_t W) of the first layer into `h` (the right-hand D^(-1/2) of the normalised adjacency is
        folded into the rows of H)."""
        with self._stage("feature_transform"):
            B.feature_transform(self.blk.x[t - 1], self.blk.weight(t, 0), h, row_scale=self.dinv[self.slot_of(t)])

    def gcn(self, t: int, h_first: Optional[torch.Tensor] = None) -> torch.Tensor:
        """All GCN layers on snapshot t; returns the frame Z_t.  h_first: the first layer's H, already formed by
        transform_first (the buffer then serves the later layers as well)."""
        blk = self.blk
        slot = self.slot_of(t)
        out = self.z[t - 1] if self.keep_all_z else self.z[0]
        h = self.h if h_first is None else h_first
        cur = blk.x[t - 1]
        for layer in range(blk.layers):
            if layer > 0 or h_first is None:
                with self._stage("feature_transform"):
                    B.feature_transform(cur, blk.weight(t, layer), h, row_scale=self.dinv[slot])
            dst = out if layer == blk.layers - 1 else self.z_mid
            with self._stage("spmm"):
                B.spmm(self.rowptr[slot], self.colidx[slot], blk.nnz[t - 1], self.dinv[slot], h, dst,
                       self.ws_spmm, flags=B.DGNN_RELU | B.DGNN_H_PRESCALED)
            cur = dst
        return out

    # A subclass whose snapshot_ready / transform_first / gcn keep to buffers that alternate with the parity of t (so
    # that the work on snapshot t+1 on the second stream never touches what the aggregation of t reads) may say so.
    two_stream_safe = True

    def begin_pass(self) -> None:
        """Called at the start of every pass (subclasses that overwrite A_1's slot reload it here)."""

    def snapshot_ready(self, t: int) -> None:
        """Called once A_t is resident (after the rebuild for t >= 2), before its GCN step."""

    def mix(self) -> None:
        """In-place M-transform over the stored frames."""
        if self.blk.window:
            with self._stage("mproduct"):
                B.mproduct(self.z, self.z, self.blk.window)

    # ------------------------------------------------------------------ whole passes
    def run_resident(self, first: int = 1, validate: bool = False, on_snapshot=None, overlap: bool = False) -> None:
        """Forward pass with the difference lists already on the device.  `first` = 2 skips the GCN
        on A_1 (timed regions that count only rebuilt snapshots).  on_snapshot(t, slot) is called
        after the work of timestep t has been enqueued.  overlap: see _run_overlapped."""
        blk = self.blk
        if overlap:
            self._run_overlapped(first, validate, on_snapshot, pinned=False, prefetch_next=False)
            return
        self.begin_pass()
        for t in range(1, blk.T + 1):
            if t >= 2:
                self.rebuild(t, blk.deltas[t - 2], validate)
            self.snapshot_ready(t)
            if t >= first:
                self.gcn(t)
            if on_snapshot is not None:
                on_snapshot(t, self.slot_of(t))
        self.mix()

    def _run_overlapped(self, first: int, validate: bool, on_snapshot, pinned: bool, prefetch_next: bool) -> None:
        """The same pass on two streams: the rebuild of A_t, whatever a subclass does to A_t (snapshot_ready) and the
        first layer's X_t W run on a second stream, up to one snapshot ahead of the aggregations on the current one.  The aggregation is held back by the rate at which
        L2 misses are served and leaves issue slots and HBM bandwidth unused, which the two streaming kernels of the
        next snapshot take.  Two H buffers alternate; A_t's slot and an H buffer are written again only after the
        aggregation that read them two snapshots earlier has finished (events both ways).  Results are those of the
        one-stream pass bit for bit: the same kernels on the same operands."""
        blk = self.blk
        assert self.two_stream_safe, "this runner enqueues work per snapshot that the two-stream pass does not know about"
        if pinned:
            assert self.stage is not None
        main = torch.cuda.current_stream(self.dev)
        if getattr(self, "prep_stream", None) is None:
            self.prep_stream = torch.cuda.Stream(device=self.dev)
            self.h_pair = [self.h, torch.empty_like(self.h)]
        prep = self.prep_stream
        self.begin_pass()                   # on the current stream, before the second one is let go
        ready = [torch.cuda.Event() for _ in range(blk.T + 1)]     # A_t, dinv_t and the first H of t are there
        done = [torch.cuda.Event() for _ in range(blk.T + 1)]      # everything that reads them has been enqueued and run

        def issue_copy(t):
            k = t % 2
            with torch.cuda.stream(self.copy_stream):
                self.copy_stream.wait_event(self.consumed[k])
                with self._stage("delta_h2d"):
                    B.delta_h2d(*blk.pinned[t - 2], *self.stage[k])
                self.copied[k].record(self.copy_stream)

        begun = torch.cuda.Event()
        begun.record(main)                  # whatever the caller enqueued before the pass (an earlier pass, load_first)
        prep.wait_event(begun)
        if pinned:
            if not getattr(self, "_first_lists_requested", False):
                for k in range(2):
                    self.consumed[k].record(main)
                if blk.T >= 2:
                    issue_copy(2)
            self._first_lists_requested = False
        for t in range(1, blk.T + 1):
            with torch.cuda.stream(prep):
                if t - 2 >= 1:
                    prep.wait_event(done[t - 2])            # A_{t-2}'s slot and its H buffer are free again
                if t >= 2:
                    if pinned:
                        k = t % 2
                        prep.wait_event(self.copied[k])
                        if t + 1 <= blk.T:
                            issue_copy(t + 1)
                        self.rebuild(t, self.stage[k], validate)
                        self.consumed[k].record(prep)
                        if t == blk.T and prefetch_next and blk.T >= 3:
                            issue_copy(2)
                            self._first_lists_requested = True
                    else:
                        self.rebuild(t, blk.deltas[t - 2], validate)
                self.snapshot_ready(t)      # a subclass's own work on A_t (it may use only what alternates with t)
                if t >= first:
                    self.transform_first(t, self.h_pair[t % 2])
                ready[t].record(prep)
            main.wait_event(ready[t])
            if t >= first:
                self.gcn(t, h_first=self.h_pair[t % 2])
            done[t].record(main)
            if on_snapshot is not None:
                on_snapshot(t, self.slot_of(t))
        self.mix()

    def capture(self, first: int = 1) -> "torch.cuda.CUDAGraph":
        """The resident pass recorded once as a HIP graph (every library call only enqueues kernels on the
        current stream, so the whole pass is capturable); replaying it costs one launch instead of one per
        kernel, which is what bounds small workloads.  The pass is run once eagerly first, so that one-time
        host-side set-up inside the library (occupancy queries) is not part of the recording."""
        self.run_resident(first=first)
        torch.cuda.synchronize(self.dev)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run_resident(first=first)
        return graph

    def run_from_pinned(self, first: int = 1, prefetch_next: bool = False, validate: bool = False, on_snapshot=None,
                        overlap: bool = False) -> None:
        """Same pass with the difference lists of step t+1 copied from pinned host memory on a second
        stream while step t computes (two staging sets, events both ways).  With prefetch_next the lists of
        the next pass's first step are already requested while this pass finishes (a stream of blocks: the
        next block's first lists travel during the current block's last steps).  on_snapshot(t, slot) as in
        run_resident; overlap: see _run_overlapped."""
        blk = self.blk
        assert self.stage is not None
        if overlap:
            self._run_overlapped(first, validate, on_snapshot, pinned=True, prefetch_next=prefetch_next)
            return
        main = torch.cuda.current_stream(self.dev)

        def issue_copy(t):
            k = t % 2
            with torch.cuda.stream(self.copy_stream):
                self.copy_stream.wait_event(self.consumed[k])
                with self._stage("delta_h2d"):           # event pair on the copy stream (the current stream here)
                    B.delta_h2d(*blk.pinned[t - 2], *self.stage[k])
                self.copied[k].record(self.copy_stream)

        if not getattr(self, "_first_lists_requested", False):
            for k in range(2):
                self.consumed[k].record(main)
            if blk.T >= 2:
                issue_copy(2)
        self._first_lists_requested = False
        self.begin_pass()
        for t in range(1, blk.T + 1):
            if t >= 2:
                k = t % 2
                main.wait_event(self.copied[k])
                if t + 1 <= blk.T:
                    issue_copy(t + 1)
                self.rebuild(t, self.stage[k], validate)
                self.consumed[k].record(main)
                if t == blk.T and prefetch_next and blk.T >= 3:     # both staging sets have been used and released
                    issue_copy(2)
                    self._first_lists_requested = True
            self.snapshot_ready(t)
            if t >= first:
                self.gcn(t)
            if on_snapshot is not None:
                on_snapshot(t, self.slot_of(t))
        self.mix()

    def snapshot_to_host(self, t: int):
        slot = self.slot_of(t)
        return self.rowptr[slot].cpu().numpy(), self.colidx[slot][: self.blk.nnz[t - 1]].cpu().numpy()


class SmoothedRunner(BlockRunner):
    """Forward pass over a block on SMOOTHED snapshots (Section "Smoothening the Input Graphs"), with the smoothing
    done on the device: the raw snapshot A_t is rebuilt from the difference lists as before, the smoothed one is
    S_t = S_{t-1} + A_t - A_{t-life} (dgnn_csr_combine on resident snapshots: a ring of life + 1 raw ones), its
    normalisation is recomputed from the weighted row sums (dgnn_csr_weighted_dinv), and the GCN step aggregates
    with the raw counts as values (dgnn_spmm_weighted with dinv).  Only the raw difference lists ever travel."""

    def __init__(self, blk: BlockInputs, life: int, keep_all_z: Optional[bool] = None, diag_value: float = 1.0):
        super().__init__(blk, keep_all_z)
        assert life >= 1
        self.life = life
        # edge-life smoothing acts on A; Eqn (1) then adds the self loop once: the stored diagonal stays 1 (0.0 here
        # leaves the summed diagonal min(life, t), which is the M-transform of the adjacency tensor instead)
        self.diag_value = diag_value
        dev, n = self.dev, blk.n
        while len(self.rowptr) < life + 1:
            self.rowptr.append(torch.empty(n + 1, dtype=torch.int32, device=dev))
            self.colidx.append(torch.empty(self.cap, dtype=torch.int32, device=dev))
            self.dinv.append(torch.empty(n, dtype=torch.float32, device=dev))
        # the window's union holds A_t and whatever the window's steps deleted
        max_del = max([int(d[2].numel()) for d in blk.deltas] + [0])
        self.cap_s = self.cap + life * max_del
        self.s = [(torch.empty(n + 1, dtype=torch.int32, device=dev), torch.empty(self.cap_s, dtype=torch.int32, device=dev),
                   torch.empty(self.cap_s, dtype=torch.float32, device=dev)) for _ in range(2)]
        self.s_nnz = 0
        self.cur = None                                 # (rowptr, colidx, val, nnz) of S_t
        self.dinv_s_pair = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(2)]   # alternate with t, like S
        self.dinv_s = self.dinv_s_pair[1]
        self.ws_combine = torch.empty(B.csr_combine_workspace(self.cap_s), dtype=torch.uint8, device=dev)
        self.ws_dinv = torch.empty(B.csr_weighted_dinv_workspace(self.cap_s), dtype=torch.uint8, device=dev)
        self.ws_spmm = torch.empty(B.spmm_workspace(n, self.cap_s, blk.f), dtype=torch.uint8, device=dev)
        self.status_s = torch.zeros(blk.T + 1, dtype=torch.int32, device=dev)   # per timestep: what dgnn_csr_combine found

    def stored_entries(self) -> int:
        """Entries of the current smoothed snapshot (reads the device: waits for the stream)."""
        return int(self.cur[0][-1])

    def slot_of(self, t: int) -> int:                   # a ring: A_{t-life} is still there when S_t is formed
        return t % (self.life + 1)

    def load_first(self) -> None:
        blk = self.blk
        slot = self.slot_of(1)
        self.rowptr[slot].copy_(blk.rowptr1)
        self.colidx[slot][: blk.nnz[0]].copy_(blk.colidx1)
        B.csr_dinv(self.rowptr[slot], self.dinv[slot])
        rp, ci, val = self.s[1]                          # S_1 = A_1, every entry counted once
        rp.copy_(blk.rowptr1)
        ci[: blk.nnz[0]].copy_(blk.colidx1)
        val[: blk.nnz[0]].fill_(1.0)
        self.cur = (rp, ci, val, blk.nnz[0])

    def smooth(self, t: int) -> None:
        """S_t from S_{t-1}, A_t and A_{t-life} (t >= 2), then its normalisation."""
        blk = self.blk
        if t >= 2:
            a_in = (self.rowptr[self.slot_of(t)], self.colidx[self.slot_of(t)], blk.nnz[t - 1])
            a_out = None
            if t - self.life >= 1:
                k = t - self.life
                a_out = (self.rowptr[self.slot_of(k)], self.colidx[self.slot_of(k)], blk.nnz[k - 1])
            out = self.s[t % 2]
            with self._stage("csr_combine"):
                B.csr_combine(self.cur, a_in, 1.0, a_out, -1.0, out, self.ws_combine, diag_value=self.diag_value,
                              status=self.status_s[t:t + 1])
            # the number of stored entries stays on the device (out[0][n]); the capacity serves as the upper bound
            self.cur = (out[0], out[1], out[2], self.cap_s)
        self.dinv_s = self.dinv_s_pair[t % 2]
        with self._stage("csr_weighted_dinv"):
            B.csr_weighted_dinv(self.cur[0], self.cur[2], self.cur[3], self.dinv_s, self.ws_dinv)

    def transform_first(self, t: int, h: torch.Tensor) -> None:
        with self._stage("feature_transform"):
            B.feature_transform(self.blk.x[t - 1], self.blk.weight(t, 0), h, row_scale=self.dinv_s_pair[t % 2])

    def gcn(self, t: int, h_first: Optional[torch.Tensor] = None) -> torch.Tensor:
        blk = self.blk
        rp, ci, val, nnz = self.cur                      # S_t as of now: the host enqueues snapshot by snapshot
        dinv_s = self.dinv_s_pair[t % 2]
        out = self.z[t - 1] if self.keep_all_z else self.z[0]
        h = self.h if h_first is None else h_first
        cur = blk.x[t - 1]
        for layer in range(blk.layers):
            if layer > 0 or h_first is None:
                with self._stage("feature_transform"):
                    B.feature_transform(cur, blk.weight(t, layer), h, row_scale=dinv_s)
            dst = out if layer == blk.layers - 1 else self.z_mid
            with self._stage("spmm_weighted"):
                B.spmm_weighted(rp, ci, val, nnz, h, dst, self.ws_spmm, flags=B.DGNN_RELU | B.DGNN_H_PRESCALED,
                                dinv=dinv_s)
            cur = dst
        return out

    def begin_pass(self) -> None:
        self.load_first()                                # the ring overwrites A_1: every pass starts from the inputs

    def snapshot_ready(self, t: int) -> None:
        self.smooth(t)
