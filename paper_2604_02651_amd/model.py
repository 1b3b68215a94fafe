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
        """params = {"W_in": d_in x d_h, "layers": [(W_l d_h x d_h, gamma_l d_h), ...], "W_out": d_h x c}: float32
        device tensors with the initial values; the live parameters are self.p (same structure), updated by step()."""
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
        f32 = dict(dtype=torch.float32, device=dev)
        self.dev, self.capacity = dev, capacity
        self._E = E

        def mat(d):   # B x d with rows starting 16-byte aligned
            return torch.empty((B, (d + 3) // 4 * 4), **f32)[:, :d]
        self._mat = mat
        self.batches = [self._new_batch()]
        self._use(self.batches[0])
        self.Xh = [mat(d_h) for _ in range(self.L + 1)]
        self.T = [mat(d_h) for _ in range(self.L)]
        self.Z = [mat(d_h) for _ in range(self.L)]
        self.inv_rms = [torch.empty(B, **f32) for _ in range(self.L)]
        self.O, self.dO = mat(c), mat(c)
        self.dX = [mat(d_h), mat(d_h)]
        self.dZ, self.dT = mat(d_h), mat(d_h)
        self.loss = torch.zeros(1, **f32)
        # Parameters, gradients and optimizer moments each live in ONE flat buffer (every tensor starting at a
        # multiple of 64 floats), so that the update is a single kernel launch; self.p / self.g are views.
        tensors = [("W_in", params["W_in"]), ("W_out", params["W_out"])]
        for l, (Wl, gl) in enumerate(params["layers"]):
            tensors += [(("layers", l, 0), Wl), (("layers", l, 1), gl)]
        offs, total = [], 0
        for _, t in tensors:
            offs.append(total)
            total += (t.numel() + 63) // 64 * 64
        self.flat_p = torch.zeros(total, **f32)
        self.flat_g = torch.zeros(total, **f32)
        views_p, views_g = [], []
        for (key, t), o in zip(tensors, offs):
            vp = self.flat_p[o:o + t.numel()].view(t.shape)
            vp.copy_(t)
            views_p.append(vp)
            views_g.append(self.flat_g[o:o + t.numel()].view(t.shape))
        self.p = {"W_in": views_p[0], "W_out": views_p[1],
                  "layers": [(views_p[2 + 2 * l], views_p[3 + 2 * l]) for l in range(self.L)]}
        self.g = {"W_in": views_g[0], "W_out": views_g[1],
                  "layers": [(views_g[2 + 2 * l], views_g[3 + 2 * l]) for l in range(self.L)]}
        if optimizer == "adam":
            self.m = torch.zeros(total, **f32)
            self.v = torch.zeros(total, **f32)
        elif optimizer not in (None, "sgd"):
            raise ValueError("optimizer must be 'adam', 'sgd' or None")

    def _new_batch(self):
        """Device buffers of one mini-batch: sample, bitmap, rank prefix, induced CSR, sliced features and labels."""
        W = (self.N + 63) // 64
        b = type("Batch", (), {})()
        b.S = torch.empty(self.B, dtype=torch.int32, device=self.dev)
        b.bitmap = torch.empty(W, dtype=torch.int64, device=self.dev)
        b.rank = torch.empty(W, dtype=torch.int32, device=self.dev)
        b.A = sg.Csr(self.B, self.B, self.capacity, self.dev)
        b.y_S = torch.empty(self.B, dtype=torch.int32, device=self.dev)
        b.X_S = self._mat(self.d_in)
        b.ready, b.free = torch.cuda.Event(), torch.cuda.Event()
        return b

    def _use(self, b):
        self.S, self.bitmap, self.rank, self.A, self.y_S, self.X_S = b.S, b.bitmap, b.rank, b.A, b.y_S, b.X_S

    # Algorithm 1, lines 1-4
    def minibatch(self, t: int, batch=None, ctx=None, stream=None):
        if batch is None:
            batch = self.batches[0]
            self._use(batch)
        b = batch
        c = ctx if ctx is not None else self.ctx
        sg.sgnn_sample_uniform(c, self.N, self.B, self.sampler_seed, t, b.S, b.bitmap, b.rank, stream=stream)
        sg.sgnn_induced_csr(c, self.N, self.rowptr, self.colidx, None, b.S, self.B, b.bitmap, b.rank, b.A, stream=stream)
        sg.sgnn_gather_rows(c, self.X, b.S, self.B, b.X_S, self.labels, b.y_S, stream=stream)

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
        if self.optimizer == "sgd":
            sg.sgnn_sgd_step(self.ctx, self.flat_p, self.flat_g, self.lr, self.weight_decay)
        else:
            sg.sgnn_adam_step(self.ctx, self.flat_p, self.flat_g, self.m, self.v, self.lr, self.t_opt)

    def step(self, t: int):
        """One training step with sampler / dropout counter t; the loss stays on the device in self.loss."""
        self._use(self.batches[0])
        self.minibatch(t)
        self.forward(t)
        self.backward(t)
        self.update()

    def run(self, steps):
        """The same steps with the mini-batch of step i+1 built on a second stream (default priority, a context
        of its own) while step i trains (Sec. V-A of the paper): two sets of mini-batch buffers, ordered by a
        ready and a free event per set.  Same results as step() one after the other, bit for bit."""
        steps = list(steps)
        if not steps:
            return
        if not hasattr(self, "side_stream"):
            self.side_stream = torch.cuda.Stream(device=self.dev)
            self.side_ctx = sg.Context(self.dev.index or 0)
            self.side_ctx.reserve(self.N, self._E, self.B, max(self.d_in, self.d_h, self.c), self.capacity)
            self.batches.append(self._new_batch())
        main, side = torch.cuda.current_stream(), self.side_stream
        start = torch.cuda.Event()
        start.record(main)
        side.wait_event(start)          # whatever used the buffers before has finished
        self.minibatch(steps[0], self.batches[0], self.side_ctx, side)
        self.batches[0].ready.record(side)
        for i, t in enumerate(steps):
            b = self.batches[i % 2]
            if i + 1 < len(steps):
                nb = self.batches[(i + 1) % 2]
                if i >= 1:
                    side.wait_event(nb.free)    # the training of step i-1 has let go of that set
                self.minibatch(steps[i + 1], nb, self.side_ctx, side)
                nb.ready.record(side)
            main.wait_event(b.ready)
            self._use(b)
            self.forward(t)
            self.backward(t)
            self.update()
            b.free.record(main)
        main.wait_stream(side)
