"""One mini-batch training step (Algorithm 1 of the paper without the parameter update) as a
sequence of libsgnn calls on preallocated device buffers.  No arithmetic happens here."""
from __future__ import annotations

from typing import List, Optional, Tuple

import torch

from . import binding as sg


class GcnStep:
    """Holds the graph, the features, the layer weights and every buffer a step needs.

    step(t) runs: sample -> induced CSR -> slice -> L x layer forward -> loss -> L x layer backward.
    With fuse_slice the feature slice X[S] is not materialised: layer 1 reads the full feature
    matrix through row_index = S, and only the labels are sliced.
    """

    def __init__(self, N: int, rowptr: torch.Tensor, colidx: torch.Tensor, X: torch.Tensor, labels: torch.Tensor,
                 weights: List[Tuple[torch.Tensor, torch.Tensor]], B: int, seed: int = 0, bf16: bool = False,
                 fuse_slice: bool = True, capacity: Optional[int] = None, device="cuda:0", ctx: Optional[sg.Context] = None,
                 auto_order: bool = True):
        self.N, self.B, self.seed = N, B, seed
        self.rowptr, self.colidx, self.X, self.labels = rowptr, colidx, X, labels
        self.weights = weights
        self.L = len(weights)
        self.flags = sg.SGNN_BF16_MFMA if bf16 else 0
        self.fuse_slice = fuse_slice
        dev = torch.device(device)
        E = int(colidx.numel())
        dims = [weights[0][0].shape[0]] + [w.shape[1] for w, _ in weights]
        self.dims = dims
        self.ctx = ctx or sg.Context(dev.index or 0)
        W = (N + 63) // 64
        self.S = torch.empty(B, dtype=torch.int32, device=dev)
        self.bitmap = torch.empty(W, dtype=torch.int64, device=dev)
        self.rank = torch.empty(W, dtype=torch.int32, device=dev)
        if capacity is None:
            # expected entries B + (E-N) B(B-1)/(N(N-1)) with generous head-room
            exp = B + (E - N) * (B / N) * ((B - 1) / max(N - 1, 1))
            capacity = int(min(E, 2 * exp + 16 * B + 65536))
        self.ctx.reserve(N, E, B, max(dims), capacity)
        self.A = sg.Csr(B, B, capacity, dev)
        self.y_S = torch.empty(B, dtype=torch.int32, device=dev)
        self.X_S = None if fuse_slice else torch.empty((B, dims[0]), dtype=torch.float32, device=dev)
        # a layer that narrows (d_out < d_in) is evaluated transform-first: its sparse products run at
        # width d_out, and its backward pass needs the layer input instead of the aggregate
        self.xform_first = [auto_order and dims[l + 1] < dims[l] for l in range(self.L)]
        self.T = [None if self.xform_first[l] else torch.empty((B, dims[l]), dtype=torch.float32, device=dev)
                  for l in range(self.L)]
        self.H = [torch.empty((B, dims[l + 1]), dtype=torch.float32, device=dev) for l in range(self.L)]
        self.dH = [torch.empty((B, dims[l]), dtype=torch.float32, device=dev) if l > 0 else None for l in range(self.L)]
        self.dO = torch.empty((B, dims[-1]), dtype=torch.float32, device=dev)
        self.dW = [torch.empty_like(w) for w, _ in weights]
        self.db = [torch.empty_like(b) for _, b in weights]
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)

    def sample(self, t: int):
        sg.sgnn_sample_uniform(self.ctx, self.N, self.B, self.seed, t, self.S, self.bitmap, self.rank)

    def induce(self):
        sg.sgnn_induced_csr(self.ctx, self.N, self.rowptr, self.colidx, None, self.S, self.B, self.bitmap, self.rank,
                            self.A)

    def slice(self):
        sg.sgnn_gather_rows(self.ctx, None if self.fuse_slice else self.X, self.S, self.B, self.X_S, self.labels,
                            self.y_S)

    def forward(self):
        for l, (W, b) in enumerate(self.weights):
            flags = self.flags | (sg.SGNN_RELU if l < self.L - 1 else 0) | (sg.SGNN_XFORM_FIRST if self.xform_first[l] else 0)
            if l == 0 and self.fuse_slice:
                sg.sgnn_gcn_fwd(self.ctx, self.A, self.X, W, b, flags, self.H[0], self.T[0], row_index=self.S)
            else:
                Hin = self.X_S if l == 0 else self.H[l - 1]
                sg.sgnn_gcn_fwd(self.ctx, self.A, Hin, W, b, flags, self.H[l], self.T[l])

    def loss_and_grad(self):
        sg.sgnn_softmax_xent(self.ctx, self.H[-1], self.y_S, self.loss, self.dO)

    def backward(self):
        dY = self.dO
        for l in range(self.L - 1, -1, -1):
            W, _ = self.weights[l]
            flags = self.flags | (sg.SGNN_RELU if l < self.L - 1 else 0) | (sg.SGNN_XFORM_FIRST if self.xform_first[l] else 0)
            saved, ridx = self.T[l], None
            if self.xform_first[l]:
                if l == 0:
                    saved, ridx = (self.X, self.S) if self.fuse_slice else (self.X_S, None)
                else:
                    saved = self.H[l - 1]
            # the induced matrix of a symmetric graph is symmetric: it is its own transpose
            sg.sgnn_gcn_bwd(self.ctx, self.A, saved, W, self.H[l], dY, flags, self.dH[l], self.dW[l], self.db[l],
                            row_index=ridx)
            dY = self.dH[l]

    def step(self, t: int):
        self.sample(t)
        self.induce()
        self.slice()
        self.forward()
        self.loss_and_grad()
        self.backward()
