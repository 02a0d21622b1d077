"""The paper's model as one object (Section 4): the encoding followed by the 64-64 ReLU network, trained with Adam on
tables and weights.  Bookkeeping only: every step of a training iteration is one call into the C-ABI library
(hashgrid_encode_mlp_fwd_train, hashgrid_loss_grad, hashgrid_mlp_bwd, hashgrid_encode_bwd[_ws], hashgrid_adam_step
twice; hashgrid_encode_bwd_input for the gradient with respect to the position); this file allocates the buffers and
keeps the step counter.

Defaults are the paper's (Section 4, "Initialization" and "Training"): tables U(-1e-4, 1e-4) in half precision behind a
full-precision master copy, Glorot-uniform weights, Adam with beta1 = 0.9, beta2 = 0.99, eps = 1e-15, an L2 factor
of 1e-6 on the network's weights only, learning rate 1e-2 (the paper: 1e-4 for signed distance functions).
"""
from __future__ import annotations

import math

import torch

from .binding import HashGrid, adam_step, loss_grad, mlp_bwd

N_HIDDEN = 64


class HashGridModel:
    def __init__(self, d: int, n_out: int, L: int = 16, F: int = 2, T: int = 1 << 19, N_min: int = 16, N_max: int = 2048,
                 loss: str = "l2", lr: float = 1e-2, l2_reg: float = 1e-6, loss_scale: float = 1.0, seed: int = 0,
                 interp: int = 0):
        """loss: "l2" or "mape".  The paper's loss is a mean over the batch; what travels backward here is the gradient
        of the summed loss times loss_scale, because the network's backward pass rounds dL/dout to half precision
        and 1/n would push it into the subnormals.  Adam is indifferent to a common factor of all gradients, and
        the L2 term of the weights gets the same factor (n * loss_scale), so the update is the mean loss's."""
        self.grid = HashGrid(d, L, F, T, N_min, N_max, "f16", "f16", interp)
        self.d, self.n_in, self.n_out = d, L * F, n_out
        self.loss, self.lr, self.l2_reg, self.loss_scale = loss, lr, l2_reg, loss_scale
        gen = torch.Generator(device="cuda").manual_seed(seed)
        n = self.grid.n_entries
        self.tables = torch.rand((n, F), device="cuda", generator=gen) * 2e-4 - 1e-4
        self.tables_half = self.tables.half()
        self._tab_grad, self._tab_m, self._tab_v = (torch.zeros_like(self.tables) for _ in range(3))
        self._shapes = [(N_HIDDEN, self.n_in), (N_HIDDEN, N_HIDDEN), (n_out, N_HIDDEN)]
        init = [(torch.rand(s, device="cuda", generator=gen) * 2 - 1) * math.sqrt(6.0 / (s[0] + s[1])) for s in self._shapes]
        self.weights = torch.cat([w.reshape(-1) for w in init]).contiguous()  # W1, W2, W3 in one array: one optimiser call
        self.weights_half = self.weights.half()
        self._net_grad, self._net_m, self._net_v = (torch.zeros_like(self.weights) for _ in range(3))
        self._W, self._dW = self._views(self.weights_half), self._views(self._net_grad)
        self.steps = 0
        self._loss_sum = torch.zeros(1, dtype=torch.float64, device="cuda")
        self._buf_B = 0

    def _views(self, flat):
        out, at = [], 0
        for r, c in self._shapes:
            out.append(flat[at:at + r * c].view(r, c))
            at += r * c
        return out

    def _buffers(self, B: int):
        if B != self._buf_B:
            self._out = torch.empty((B, self.n_out), device="cuda")
            self._dout = torch.empty_like(self._out)
            self._y = torch.empty((B, self.n_in), dtype=torch.float16, device="cuda")
            self._dy = torch.empty_like(self._y)
            self._buf_B = B

    def infer(self, x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """The network's output [B, n_out] fp32 for points x [B, d] in [0,1)^d."""
        return self.grid.encode_mlp_fwd(x, self.tables_half, *self._W, out)

    def input_gradient(self, x: torch.Tensor, dLdout: torch.Tensor | None = None) -> torch.Tensor:
        """d(sum_i dLdout_i * out_i) / dx [B, d] fp32: with the default dLdout = 1 and one output, the gradient of the
        output with respect to the position (the normal of a signed distance function, Section 3: the encoding is
        continuous and its derivative piecewise constant).  Three calls: the fused forward keeping y, the network's
        backward pass (its weight gradients go to a scratch array), hashgrid_encode_bwd_input."""
        B = x.shape[0]
        self._buffers(B)
        self.grid.encode_mlp_fwd(x, self.tables_half, *self._W, self._out, y=self._y)
        if dLdout is None:
            dLdout = torch.ones((B, self.n_out), device="cuda")
        if not hasattr(self, "_dW_scratch"):
            self._dW_scratch = self._views(torch.zeros_like(self._net_grad))
        mlp_bwd(self._y, *self._W, dLdout, self._dy, *self._dW_scratch)
        return self.grid.encode_bwd_input(x, self.tables_half, self._dy)

    def step(self, x: torch.Tensor, target: torch.Tensor) -> None:
        """One training iteration on the batch (x [B, d], target [B, n_out], fp32 device tensors).  Nothing here
        synchronises; last_loss() does."""
        B = x.shape[0]
        self._buffers(B)
        self.steps += 1
        self.grid.encode_mlp_fwd(x, self.tables_half, *self._W, self._out, y=self._y)
        self._loss_sum.zero_()
        loss_grad(self._out, target, self.loss, self.loss_scale, self._dout, self._loss_sum)
        self._n_last = B * self.n_out
        mlp_bwd(self._y, *self._W, self._dout, self._dy, *self._dW)
        self.grid.encode_bwd(x, self._dy, self._tab_grad, overwrite=True)
        adam_step(self.tables, self._tab_grad, self._tab_m, self._tab_v, self.steps, lr=self.lr,
                  params_half=self.tables_half, zero_grad=False)
        adam_step(self.weights, self._net_grad, self._net_m, self._net_v, self.steps, lr=self.lr,
                  params_half=self.weights_half, zero_grad=True, l2_reg=self.l2_reg * self.loss_scale * self._n_last)

    def last_loss(self) -> float:
        """Mean loss over the scalars of the last step's batch, before that step's update (synchronises)."""
        return float(self._loss_sum.cpu()[0]) / self._n_last
