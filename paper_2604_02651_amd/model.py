"""The paper's complete model on the C-ABI library (Fig. 2; Sec. III-B forward, Sec. III-C backward):

    X_h0 = X_S W_in;   for l = 1..L:  T_l = A X_h,l-1,  Z_l = T_l W_l,
    X_h,l = dropout(relu(rmsnorm(Z_l; gamma_l))) + X_h,l-1;   O = X_h,L W_out;   mean cross-entropy,

one mini-batch training step = Algorithm 1: sample, induced subgraph, slice, forward, loss, backward
with the transposed matrix, parameter update.  This module only strings library calls together on
preallocated device buffers; every product, the layer tail, the loss and the update run in the HIP
kernels of libsgnn.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import torch

from . import binding as sg


class ScaleGnnModel:
    def __init__(self, N: int, rowptr: torch.Tensor, colidx: torch.Tensor, X: torch.Tensor, labels: torch.Tensor,
                 params: Dict, B: int, sampler_seed: int = 0, drop_q: float = 0.0, drop_seed: int = 1, eps: float = 1e-6,
                 bf16: bool = False, optimizer: Optional[str] = "adam", lr: float = 1e-2, weight_decay: float = 0.0,
                 capacity: Optional[int] = None, device="cuda:0", ctx: Optional[sg.Context] = None):
        """params = {"W_in": d_in x d_h, "layers": [(W_l d_h x d_h, gamma_l d_h), ...], "W_out": d_h x c}: contiguous
        float32 device tensors, updated in place by step()."""
        self.N, self.B = N, B
        self.rowptr, self.colidx, self.X, self.labels = rowptr, colidx, X, labels
        self.p = params
        self.L = len(params["layers"])
        d_in, d_h = params["W_in"].shape
        c = params["W_out"].shape[1]
        self.d_in, self.d_h, self.c = d_in, d_h, c
        self.sampler_seed, self.drop_q, self.drop_seed, self.eps = sampler_seed, drop_q, drop_seed, eps
        self.flags = sg.SGNN_BF16_MFMA if bf16 else 0
        self.optimizer, self.lr, self.weight_decay = optimizer, lr, weight_decay
        self.t_opt = 0
        dev = torch.device(device)
        self.ctx = ctx if ctx is not None else sg.Context(dev.index or 0)
        E = int(colidx.numel())
        if capacity is None:
            p = (B - 1) / max(N - 1, 1)
            capacity = int(min(E, 2 * (E * p * p + B) + 16 * B + 65536))
        self.ctx.reserve(N, E, B, max(d_in, d_h, c), capacity)
        W = (N + 63) // 64
        f32 = dict(dtype=torch.float32, device=dev)
        self.S = torch.empty(B, dtype=torch.int32, device=dev)
        self.bitmap = torch.empty(W, dtype=torch.int64, device=dev)
        self.rank = torch.empty(W, dtype=torch.int32, device=dev)
        self.A = sg.Csr(B, B, capacity, dev)
        self.y_S = torch.empty(B, dtype=torch.int32, device=dev)

        def mat(d):   # B x d with rows starting 16-byte aligned
            return torch.empty((B, (d + 3) // 4 * 4), **f32)[:, :d]
        self.X_S = mat(d_in)
        self.Xh = [mat(d_h) for _ in range(self.L + 1)]
        self.T = [mat(d_h) for _ in range(self.L)]
        self.Z = [mat(d_h) for _ in range(self.L)]
        self.inv_rms = [torch.empty(B, **f32) for _ in range(self.L)]
        self.O, self.dO = mat(c), mat(c)
        self.dX = [mat(d_h), mat(d_h)]
        self.dZ, self.dT = mat(d_h), mat(d_h)
        self.loss = torch.zeros(1, **f32)
        self.g = {"W_in": torch.empty_like(params["W_in"]), "W_out": torch.empty_like(params["W_out"]),
                  "layers": [(torch.empty_like(Wl), torch.empty_like(gl)) for Wl, gl in params["layers"]]}
        self._pairs: List[Tuple[torch.Tensor, torch.Tensor]] = [(params["W_in"], self.g["W_in"]), (params["W_out"], self.g["W_out"])]
        for (Wl, gl), (dWl, dgl) in zip(params["layers"], self.g["layers"]):
            self._pairs += [(Wl, dWl), (gl, dgl)]
        if optimizer == "adam":
            self.m = [torch.zeros_like(w) for w, _ in self._pairs]
            self.v = [torch.zeros_like(w) for w, _ in self._pairs]
        elif optimizer not in (None, "sgd"):
            raise ValueError("optimizer must be 'adam', 'sgd' or None")

    # Algorithm 1, lines 1-4
    def minibatch(self, t: int):
        c = self.ctx
        sg.sgnn_sample_uniform(c, self.N, self.B, self.sampler_seed, t, self.S, self.bitmap, self.rank)
        sg.sgnn_induced_csr(c, self.N, self.rowptr, self.colidx, None, self.S, self.B, self.bitmap, self.rank, self.A)
        sg.sgnn_gather_rows(c, self.X, self.S, self.B, self.X_S, self.labels, self.y_S)

    # line 5 (Sec. III-B)
    def forward(self, t: int):
        c, f = self.ctx, self.flags
        sg.sgnn_gemm(c, False, False, self.X_S, self.p["W_in"], None, f, self.Xh[0])
        for l, (W, gam) in enumerate(self.p["layers"]):
            sg.sgnn_spmm(c, self.A, self.Xh[l], self.T[l])                                    # Eq. 5
            sg.sgnn_gemm_tail_fwd(c, self.T[l], W, gam, self.eps, self.Xh[l], self.drop_q, self.drop_seed, l, t, f,
                                  self.Z[l], self.Xh[l + 1], self.inv_rms[l])                 # Eqs. 6-10
        sg.sgnn_gemm(c, False, False, self.Xh[self.L], self.p["W_out"], None, f, self.O)

    # lines 6-7 (Sec. III-C); the induced matrix of a symmetric graph is its own transpose
    def backward(self, t: int):
        c, f = self.ctx, self.flags
        sg.sgnn_softmax_xent(c, self.O, self.y_S, self.loss, self.dO)
        sg.sgnn_gemm(c, True, False, self.Xh[self.L], self.dO, None, f, self.g["W_out"])
        cur = 0
        sg.sgnn_gemm(c, False, True, self.dO, self.p["W_out"], None, f, self.dX[cur])
        for l in range(self.L - 1, -1, -1):
            W, gam = self.p["layers"][l]
            dW, dgam = self.g["layers"][l]
            sg.sgnn_tail_bwd(c, self.Z[l], self.inv_rms[l], gam, self.drop_q, self.drop_seed, l, t, self.dX[cur], self.dZ,
                             dgam, None)
            sg.sgnn_gemm(c, True, False, self.T[l], self.dZ, None, f, dW)                     # grad W_l
            sg.sgnn_gemm(c, False, True, self.dZ, W, None, f, self.dT)                        # grad H_agg
            sg.sgnn_spmm(c, self.A, self.dT, self.dX[1 - cur], add=self.dX[cur])              # A^T grad + skip path
            cur = 1 - cur
        self.dXh0 = self.dX[cur]
        sg.sgnn_gemm(c, True, False, self.X_S, self.dXh0, None, f, self.g["W_in"])

    def update(self):
        if self.optimizer is None:
            return
        self.t_opt += 1
        for i, (w, g) in enumerate(self._pairs):
            if self.optimizer == "sgd":
                sg.sgnn_sgd_step(self.ctx, w, g, self.lr, self.weight_decay)
            else:
                sg.sgnn_adam_step(self.ctx, w, g, self.m[i], self.v[i], self.lr, self.t_opt)

    def step(self, t: int):
        """One training step with sampler / dropout counter t; the loss stays on the device in self.loss."""
        self.minibatch(t)
        self.forward(t)
        self.backward(t)
        self.update()
