"""Caller-side plumbing for the forward pass of one CD-GCN layer over a block of timesteps (Section "CD-GCN"):
per snapshot the GCN operation with skip connection, then one LSTM step per vertex,

    Y0 = A~_t X_t           dgnn_spmm (no ReLU) on rows pre-scaled by dinv      Y1 = Y0 W      dgnn_feature_transform
    Y  = relu(Y0 o Y1)      dgnn_concat_relu
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
        with self._stage("feature_transform"):
            B.feature_transform(self.y0, self.w, self.y1)
        with self._stage("concat_relu"):
            B.concat_relu(self.y0, self.y1, self.y)
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

    def run(self) -> torch.Tensor:
        """The whole block from the initial state (h, c) = 0; returns h_t for t = 1..T."""
        blk = self.blk
        self.c.zero_()
        for t in range(1, blk.T + 1):
            if t >= 2:
                self.rebuild(t, blk.deltas[t - 2])
            self.step(t)
        return self.h_all
