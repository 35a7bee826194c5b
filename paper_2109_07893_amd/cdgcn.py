"""Caller-side plumbing for the forward pass of one CD-GCN layer over a block of timesteps (Section "CD-GCN"):
per snapshot the GCN operation with skip connection, then one LSTM step per vertex,

    Y0 = A~_t X_t           dgnn_spmm (no ReLU) on rows pre-scaled by dinv      Y1 = Y0 W      dgnn_feature_transform
    Y  = relu(Y0 o Y1)      dgnn_concat_relu           (both in one pass where the widths allow: dgnn_transform_concat_relu)
    a  = Y W_x + h W_h + b  two dgnn_feature_transform     (h, c) <- LSTM cell      dgnn_lstm_cell

Buffers and call order only; the arithmetic is in the HIP kernels."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B
from .pipeline import BlockInputs, BlockRunner


class CdgcnLayer(BlockRunner):
    """Reuses the runner's snapshot slots and rebuilds; `hidden` is the LSTM state width (4 * hidden and
    blk.f + f_out must be feature widths the dense transform takes)."""

    two_stream_safe = False       # the layer's own pass is run(); its buffers do not alternate with t

    def __init__(self, blk: BlockInputs, w: torch.Tensor, w_x: torch.Tensor, w_h: torch.Tensor,
                 bias: Optional[torch.Tensor], hidden: int, fused: bool = True):
        super().__init__(blk, keep_all_z=False)
        self.fused = fused            # one-kernel LSTM step where the library has it (fp32, hidden 32)
        n, f = blk.n, blk.f
        f_out = w.shape[1]
        dt, dev = blk.x[0].dtype, self.dev
        self.w, self.w_x, self.w_h, self.bias, self.hidden = w, w_x, w_h, bias, hidden
        assert tuple(w_x.shape) == (f + f_out, 4 * hidden) and tuple(w_h.shape) == (hidden, 4 * hidden)
        # the right-hand D^(-1/2) of A~ is folded into the rows of X by the dense transform with W = I, so that the
        # aggregation gathers rows only (twice as fast as gathering dinv per entry as well)
        self.eye = torch.eye(f, dtype=dt, device=dev)
        self.xs = torch.empty((n, f), dtype=dt, device=dev)
        self.y0 = torch.empty((n, f), dtype=dt, device=dev)
        self.y1 = torch.empty((n, f_out), dtype=dt, device=dev)
        self.y = torch.empty((n, f + f_out), dtype=dt, device=dev)
        self.gx = torch.empty((n, 4 * hidden), dtype=dt, device=dev)
        self.gh = torch.empty((n, 4 * hidden), dtype=dt, device=dev)
        self.c = torch.zeros((n, hidden), dtype=dt, device=dev)
        self.h_all = torch.empty((blk.T, n, hidden), dtype=dt, device=dev)      # h_t for every timestep
        self.h0 = torch.zeros((n, hidden), dtype=dt, device=dev)

    def step(self, t: int) -> None:
        blk = self.blk
        slot = self.slot_of(t)
        with self._stage("row_scale"):
            B.feature_transform(blk.x[t - 1], self.eye, self.xs, row_scale=self.dinv[slot])
        with self._stage("spmm"):
            B.spmm(self.rowptr[slot], self.colidx[slot], blk.nnz[t - 1], self.dinv[slot], self.xs, self.y0, self.ws_spmm,
                   flags=B.DGNN_H_PRESCALED)
        self.form_y()
        h_prev = self.h0 if t == 1 else self.h_all[t - 2]
        if self.fused and B.lstm_step_supported(self.y, self.hidden):
            with self._stage("lstm_step"):
                B.lstm_step(self.y, h_prev, self.w_x, self.w_h, self.bias, self.c, self.h_all[t - 1])
            return
        with self._stage("feature_transform"):
            B.feature_transform(self.y, self.w_x, self.gx)
            B.feature_transform(h_prev, self.w_h, self.gh)
        with self._stage("lstm_cell"):
            B.lstm_cell(self.gx, self.gh, self.bias, self.c, self.c, self.h_all[t - 1])

    def form_y(self) -> None:
        """Y = relu(Y0 o Y0 W) from self.y0: one kernel where the library has it, else the product and the concatenation."""
        if self.fused and B.transform_concat_relu_supported(self.y0, self.w.shape[1]):
            with self._stage("transform_concat_relu"):
                B.transform_concat_relu(self.y0, self.w, self.y)
            return
        with self._stage("feature_transform"):
            B.feature_transform(self.y0, self.w, self.y1)
        with self._stage("concat_relu"):
            B.concat_relu(self.y0, self.y1, self.y)

    def run(self) -> torch.Tensor:
        """The whole block from the initial state (h, c) = 0; returns h_t for t = 1..T."""
        blk = self.blk
        self.c.zero_()
        for t in range(1, blk.T + 1):
            if t >= 2:
                self.rebuild(t, blk.deltas[t - 2])
            self.step(t)
        return self.h_all


class CdgcnTrainer(CdgcnLayer):
    """Forward and backward over one block for the CD-GCN layer (Section "CD-GCN", trained as in Section "Gradient
    Checkpoint": the forward pass keeps only the LSTM states (h_t, c_t) of every timestep; the backward pass walks
    the snapshots in reverse (rebuilds with the two lists exchanged) and recomputes each timestep's GCN operation
    and gate pre-activations before taking their adjoints):

        t = T..1:  recompute Y0, Y1, Y, a_x = Y W_x, a_h = h_{t-1} W_h
                   (da, dc_{t-1}) <- LSTM cell backward of (G_t + dh_t, dc_t)        dgnn_lstm_cell_backward
                   dW_x += Y^T da, dW_h += h_{t-1}^T da, db += colsum(da)            dgnn_weight_grad, dgnn_bias_grad
                   dY = da W_x^T, dh_{t-1} = da W_h^T                                dgnn_input_grad
                   dY1 = (dY where Y > 0)[:, F:]                                     dgnn_concat_relu_backward
                   dW += Y0^T dY1                                                    dgnn_weight_grad

    Gradients with respect to the layer's parameters (fp32): dw, dw_x, dw_h, db.  The input features are leaves."""

    def __init__(self, blk: BlockInputs, w, w_x, w_h, bias, hidden: int, fused: bool = True, keep_activations: bool = False,
                 want_dx: bool = False, transposed_first=None, transposed_deltas=None):
        super().__init__(blk, w, w_x, w_h, bias, hidden, fused)
        # want_dx: also dL/dX_t = A~_t^T (dY0 + dY1 W^T), for a layer that lies below (the paper stacks two of these
        # layers).  For a directed workload that takes the transposed snapshots, a second chain rebuilt from the
        # difference lists sorted by (col, row), handed in as (rowptr, colidx) of A_1^T and one list tuple per step.
        self.want_dx = want_dx
        self.at = None
        if want_dx:
            from .training import _Chain
            self.dx = torch.empty((blk.T, blk.n, blk.f), dtype=blk.x[0].dtype, device=self.dev)
            self.d0 = torch.empty((blk.n, blk.f), dtype=blk.x[0].dtype, device=self.dev)
            self.tmp = torch.empty((blk.n, blk.f), dtype=blk.x[0].dtype, device=self.dev)
            if transposed_first is not None:
                self.at = _Chain(blk.n, self.cap, self.dev, transposed_first[0], transposed_first[1], with_dinv=False)
                self.t_deltas = transposed_deltas
        n, f, T = blk.n, blk.f, blk.T
        f_out = w.shape[1]
        dt, dev = blk.x[0].dtype, self.dev
        # With keep_activations the forward pass also keeps Y0 and Y of every timestep (N x (2F + F') per step: 6.4 GB
        # at c5's size, a matter of course in 288 GB) and the backward pass neither recomputes the GCN operation
        # nor needs the snapshots again; without, only the LSTM states are kept, as gradient checkpointing has it.
        self.keep = keep_activations
        if keep_activations:
            self.y0_all = torch.empty((T, n, f), dtype=dt, device=dev)
            self.y_all = torch.empty((T, n, f + f_out), dtype=dt, device=dev)
        self.c_all = torch.zeros((T + 1, n, hidden), dtype=dt, device=dev)     # c_0 = 0, c_t after step t
        self.da = torch.empty((n, 4 * hidden), dtype=dt, device=dev)
        self.dy = torch.empty((n, f + f_out), dtype=dt, device=dev)
        self.dy1 = torch.empty((n, f_out), dtype=dt, device=dev)
        self.dh = torch.empty((n, hidden), dtype=dt, device=dev)
        self.dc = torch.empty((n, hidden), dtype=dt, device=dev)
        self.dw = torch.zeros((f, f_out), dtype=torch.float32, device=dev)
        self.dw_x = torch.zeros((f + f_out, 4 * hidden), dtype=torch.float32, device=dev)
        self.dw_h = torch.zeros((hidden, 4 * hidden), dtype=torch.float32, device=dev)
        self.db = torch.zeros(4 * hidden, dtype=torch.float32, device=dev)
        need = max(B.weight_grad_workspace(f + f_out, 4 * hidden), B.weight_grad_workspace(hidden, 4 * hidden),
                   B.weight_grad_workspace(f, f_out))
        self.ws_wgrad = torch.empty(need, dtype=torch.uint8, device=dev)
        self.ws_bias = torch.empty(B.bias_grad_workspace(4 * hidden), dtype=torch.uint8, device=dev)

    def _gcn(self, t: int) -> None:
        """Y0, Y1 and Y of timestep t (A_t resident in its slot)."""
        blk = self.blk
        slot = self.slot_of(t)
        with self._stage("row_scale"):
            B.feature_transform(blk.x[t - 1], self.eye, self.xs, row_scale=self.dinv[slot])
        with self._stage("spmm"):
            B.spmm(self.rowptr[slot], self.colidx[slot], blk.nnz[t - 1], self.dinv[slot], self.xs, self.y0, self.ws_spmm,
                   flags=B.DGNN_H_PRESCALED)
        self.form_y()

    def forward(self) -> torch.Tensor:
        blk = self.blk
        self.c_all[0].zero_()
        for t in range(1, blk.T + 1):
            if t >= 2:
                self.rebuild(t, blk.deltas[t - 2])
                if self.at is not None:
                    self._rebuild_transposed(t - 1, t, blk.nnz[t - 2], reverse=False)
            if self.keep:
                self.y0, self.y = self.y0_all[t - 1], self.y_all[t - 1]
            self._gcn(t)
            h_prev = self.h0 if t == 1 else self.h_all[t - 2]
            if self.fused and B.lstm_step_supported(self.y, self.hidden):
                with self._stage("lstm_step"):          # the fused step updates the cell state in place
                    self.c_all[t].copy_(self.c_all[t - 1])
                    B.lstm_step(self.y, h_prev, self.w_x, self.w_h, self.bias, self.c_all[t], self.h_all[t - 1])
                continue
            with self._stage("feature_transform"):
                B.feature_transform(self.y, self.w_x, self.gx)
                B.feature_transform(h_prev, self.w_h, self.gh)
            with self._stage("lstm_cell"):
                B.lstm_cell(self.gx, self.gh, self.bias, self.c_all[t - 1], self.c_all[t], self.h_all[t - 1])
        return self.h_all

    def _rebuild_transposed(self, src_t: int, dst_t: int, nnz_src: int, reverse: bool) -> None:
        ar, ac, dr, dc = self.t_deltas[max(src_t, dst_t) - 2]
        if reverse:
            ar, ac, dr, dc = dr, dc, ar, ac
        a = self.at
        s, d = a.slot_of(src_t), a.slot_of(dst_t)
        with self._stage("delta_rebuild"):
            B.delta_rebuild(a.rowptr[s], a.colidx[s], nnz_src, ar, ac, int(ar.numel()), dr, dc, int(dr.numel()),
                            a.rowptr[d], a.colidx[d], None, self.ws_rebuild)

    def backward(self, g_h: torch.Tensor) -> None:
        """g_h [T, n, hidden] = dL/dh_t.  Must follow forward() (A_T resident)."""
        blk = self.blk
        T = blk.T
        first = True
        for t in range(T, 0, -1):
            if self.keep:
                self.y0, self.y = self.y0_all[t - 1], self.y_all[t - 1]
            else:
                self._gcn(t)
            h_prev = self.h0 if t == 1 else self.h_all[t - 2]
            carried = (None, None) if t == T else (self.dh, self.dc)
            if self.fused and B.lstm_step_backward_supported(self.y, self.hidden):
                with self._stage("lstm_step_backward"):
                    B.lstm_step_backward(self.y, h_prev, self.w_x, self.w_h, self.bias, self.c_all[t - 1], g_h[t - 1],
                                         carried[0], carried[1], self.da, self.dc)
            else:
                with self._stage("feature_transform"):
                    B.feature_transform(self.y, self.w_x, self.gx)
                    B.feature_transform(h_prev, self.w_h, self.gh)
                with self._stage("lstm_cell_backward"):
                    B.lstm_cell_backward(self.gx, self.gh, self.bias, self.c_all[t - 1], g_h[t - 1], carried[0], carried[1],
                                         self.da, self.dc)
            with self._stage("weight_grad"):
                B.weight_grad(self.y, self.da, self.dw_x, self.ws_wgrad, accumulate=not first)
                B.weight_grad(h_prev, self.da, self.dw_h, self.ws_wgrad, accumulate=not first)
            with self._stage("bias_grad"):
                B.bias_grad(self.da, self.db, self.ws_bias, accumulate=not first)
            with self._stage("input_grad"):
                B.input_grad(self.da, self.w_x, self.dy)
                if t >= 2:
                    B.input_grad(self.da, self.w_h, self.dh)
            with self._stage("concat_relu_backward"):
                B.concat_relu_backward(self.dy, self.y, self.d0 if self.want_dx else None, self.dy1, blk.f)
            with self._stage("weight_grad"):
                B.weight_grad(self.y0, self.dy1, self.dw, self.ws_wgrad, accumulate=not first)
            if self.want_dx:
                slot = self.slot_of(t)
                with self._stage("input_grad"):
                    B.input_grad(self.dy1, self.w, self.tmp)
                    B.add(self.d0, self.tmp, self.d0)                           # dY0: its own block and the path through Y1
                with self._stage("row_scale"):
                    B.feature_transform(self.d0, self.eye, self.tmp, row_scale=self.dinv[slot])
                with self._stage("spmm_transposed"):
                    rp, ci = ((self.at.rowptr[slot], self.at.colidx[slot]) if self.at is not None
                              else (self.rowptr[slot], self.colidx[slot]))
                    B.spmm(rp, ci, blk.nnz[t - 1], self.dinv[slot], self.tmp, self.dx[t - 1], self.ws_spmm,
                           flags=B.DGNN_H_PRESCALED)
                if t >= 3 and self.at is not None:
                    self._rebuild_transposed(t, t - 1, blk.nnz[t - 1], reverse=True)
            first = False
            if t >= 3 and (self.want_dx or not self.keep):      # A_{t-1} from A_t: the two lists exchanged (A_1 was kept)
                ar, ac, dr, dc = blk.deltas[t - 2]
                src, dst = self.slot_of(t), self.slot_of(t - 1)
                with self._stage("delta_rebuild"):
                    B.delta_rebuild(self.rowptr[src], self.colidx[src], blk.nnz[t - 1], dr, dc, int(dr.numel()), ar, ac,
                                    int(ar.numel()), self.rowptr[dst], self.colidx[dst], self.dinv[dst], self.ws_rebuild)
