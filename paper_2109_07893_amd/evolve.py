"""Caller-side plumbing for EvolveGCN's weights (Section "EvolveGCN"): the GCN weight of timestep t comes from the
one before through an LSTM, W_t = LSTM(W_{t-1}).  Reading (the section gives only that line; this is the variant
it names, EGCN-O): the weight matrix is the LSTM's hidden state AND its input, its F rows are the batch, and a cell
state C of the same shape is carried along,

    a_t = W_{t-1} U_x + W_{t-1} U_h + b,    (W_t, C_t) = cell(a_t, C_{t-1})          W_0 given, C_0 = 0.

The matrices are F x F', so all of this is a handful of tiny launches of the same kernels the CD-GCN layer uses
(dgnn_feature_transform, dgnn_lstm_cell and, going back, dgnn_lstm_cell_backward, dgnn_weight_grad,
dgnn_input_grad, dgnn_bias_grad, dgnn_add).  fp32, 4 F' <= 128.  Buffers and call order only."""
from __future__ import annotations

from typing import List

import torch

from . import binding as B


class EvolvingWeights:
    def __init__(self, w0: torch.Tensor, u_x: torch.Tensor, u_h: torch.Tensor, bias: torch.Tensor, T: int):
        f, f2 = w0.shape
        assert w0.dtype == torch.float32 and tuple(u_x.shape) == (f2, 4 * f2) and tuple(u_h.shape) == (f2, 4 * f2)
        dev = w0.device
        self.w0, self.u_x, self.u_h, self.bias, self.T = w0, u_x, u_h, bias, T
        self.w = torch.empty((T, f, f2), device=dev)              # W_1 .. W_T
        self.c = torch.zeros((T + 1, f, f2), device=dev)          # C_0 = 0, C_t
        self.gx = torch.empty((f, 4 * f2), device=dev)
        self.gh = torch.empty((f, 4 * f2), device=dev)
        self.da = torch.empty((f, 4 * f2), device=dev)
        self.dh = torch.empty((f, f2), device=dev)
        self.dh2 = torch.empty((f, f2), device=dev)
        self.dc = torch.empty((f, f2), device=dev)
        self.du_x = torch.zeros((f2, 4 * f2), device=dev)
        self.du_h = torch.zeros((f2, 4 * f2), device=dev)
        self.db = torch.zeros(4 * f2, device=dev)
        self.dw0 = torch.empty((f, f2), device=dev)
        self.ws_wgrad = torch.empty(B.weight_grad_workspace(f2, 4 * f2), dtype=torch.uint8, device=dev)
        self.ws_bias = torch.empty(B.bias_grad_workspace(4 * f2), dtype=torch.uint8, device=dev)

    def _prev(self, t: int) -> torch.Tensor:
        return self.w0 if t == 1 else self.w[t - 2]

    def _gates(self, t: int) -> None:
        B.feature_transform(self._prev(t), self.u_x, self.gx)
        B.feature_transform(self._prev(t), self.u_h, self.gh)

    def forward(self) -> List[torch.Tensor]:
        """W_1 .. W_T (views of one buffer)."""
        for t in range(1, self.T + 1):
            self._gates(t)
            B.lstm_cell(self.gx, self.gh, self.bias, self.c[t - 1], self.c[t], self.w[t - 1])
        return [self.w[t] for t in range(self.T)]

    def backward(self, dw_t: List[torch.Tensor]) -> None:
        """dw_t[t-1] = dL/dW_t (fp32, from the GCN steps).  Leaves dL/dU_x, dL/dU_h, dL/db and dL/dW_0."""
        for t in range(self.T, 0, -1):
            self._gates(t)                                         # recomputed, as everywhere in the backward pass
            last = t == self.T
            B.lstm_cell_backward(self.gx, self.gh, self.bias, self.c[t - 1], dw_t[t - 1], None if last else self.dh,
                                 None if last else self.dc, self.da, self.dc)
            B.weight_grad(self._prev(t), self.da, self.du_x, self.ws_wgrad, accumulate=not last)
            B.weight_grad(self._prev(t), self.da, self.du_h, self.ws_wgrad, accumulate=not last)
            B.bias_grad(self.da, self.db, self.ws_bias, accumulate=not last)
            # W_{t-1} feeds both products
            B.input_grad(self.da, self.u_x, self.dh)
            B.input_grad(self.da, self.u_h, self.dh2)
            B.add(self.dh, self.dh2, self.dh)
        self.dw0.copy_(self.dh)
