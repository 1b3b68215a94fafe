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
                 auto_order: bool = True, fuse_relu_bwd: bool = True, side_dw: bool = False, bf16_activations: bool = False,
                 pad_features: bool = True, bf16_loss_grad: bool = True, fuse_loss: bool = False, keep_logits: bool = True):
        """bf16_activations (with bf16): the aggregates T_l and the layer outputs H_l (all but the logits) are stored as
        bfloat16, and so is the gradient dH_l handed to an aggregate-first layer below whose ReLU backward is fused
        upstream (only dense products, which round it to bfloat16 anyway, read it); the loss gradient dO is stored as
        bfloat16 as well; every other gradient handed between calls stays fp32."""
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
        if capacity is None:
            # expected entries B + (E-N) B(B-1)/(N(N-1)) with generous head-room
            exp = B + (E - N) * (B / N) * ((B - 1) / max(N - 1, 1))
            capacity = int(min(E, 2 * exp + 16 * B + 65536))
        self.capacity = capacity
        self.ctx.reserve(N, E, B, max(max(dims), (dims[0] + 31) // 32 * 32), capacity)   # a padded first layer included
        self.dev = dev
        self.batches = [self._new_batch()]
        self._use(self.batches[0])
        # a layer that narrows (d_out < d_in) is evaluated transform-first: its sparse products run at
        # width d_out, and its backward pass needs the layer input instead of the aggregate
        self.xform_first = [auto_order and dims[l + 1] < dims[l] for l in range(self.L)]
        if X.dtype == torch.bfloat16 and (not fuse_slice or self.xform_first[0]):
            raise ValueError("bfloat16 features are read by the first layer's sparse product only: they need fuse_slice "
                             "and a first layer that aggregates first")
        # A transform-first first layer multiplies X[S] by W_1 and X[S]^T by dP: with fp32 operands both go through
        # the direct-to-LDS kernels, which copy whole 32-column slices of 16-byte aligned rows.  A feature width that is
        # not a multiple of 32 (602) is therefore padded with zero columns, in a copy of X made once here, and W_1 / dW_1
        # live in buffers with as many zero rows; weights[0][0] and dW[0] are views of their first d_in rows.
        self.d_in_padded = dims[0]
        if pad_features and self.xform_first[0] and fuse_slice and not bf16 and X.dtype == torch.float32 and dims[0] % 32:
            dp = (dims[0] + 31) // 32 * 32
            Xp = torch.zeros((N, dp), dtype=torch.float32, device=dev)
            Xp[:, :dims[0]] = X
            Wp = torch.zeros((dp, dims[1]), dtype=torch.float32, device=dev)
            Wp[:dims[0]] = weights[0][0]
            self.X, self.d_in_padded = Xp, dp
            self._W0 = Wp
            self.weights = [(Wp[:dims[0]], weights[0][1])] + list(weights[1:])
        self.fuse_relu_bwd = fuse_relu_bwd
        self.side_dw = side_dw      # run() / graphs: weight-gradient GEMMs on the second stream
        if bf16_activations and not bf16:
            raise ValueError("bfloat16 storage of the activations goes with bfloat16 GEMM operands (bf16=True)")
        self.bf16_activations = bf16_activations
        act = torch.bfloat16 if bf16_activations else torch.float32
        def mat(d, dtype=torch.float32):   # B x d with every row starting on a 64-byte boundary (rows that straddle them are
            pad = 32 if dtype == torch.bfloat16 else 16     # written as partial segments: 172 fp32 columns cost 514 us against 350)
            return torch.empty((B, (d + pad - 1) // pad * pad), dtype=dtype, device=dev)[:, :d]
        self.T = [None if self.xform_first[l] else mat(dims[l], act) for l in range(self.L)]
        self.H = [mat(dims[l + 1], act if l < self.L - 1 else torch.float32) for l in range(self.L)]
        # dH[l] is the dY of layer l-1: bfloat16 when that layer reads it in its dense products only
        def dh_type(l):
            below_ok = not self.xform_first[l - 1] and fuse_relu_bwd
            return act if (bf16_activations and below_ok) else torch.float32
        self.dH = [mat(dims[l], dh_type(l)) if l > 0 else None for l in range(self.L)]
        # the loss gradient: bfloat16 along with the activations (the last layer has no ReLU, so whichever product reads
        # it - dense or sparse - takes the stored values as they are; its bias gradient comes with the loss kernel)
        self.dO = mat(dims[-1], act if bf16_loss_grad else torch.float32)
        # A transform-first last layer ends in the sparse product O = A (H W) + b, whose wavefronts hold whole rows of
        # logits: with fuse_loss the loss and its gradient are formed right there (sgnn_spmm_xent) instead of reading O
        # back in a kernel of its own; keep_logits = False does not even write O (H[-1] then keeps stale values).
        # The row epilogue costs the sparse kernel most of what the separate loss kernel costs (a row occupies 43 of
        # a wavefront's 64 lanes for 172 classes): +2 % at 2^20 rows, nothing at 2^18, a loss on dense mini-batches whose
        # long rows add their share through atomics.  Off unless asked for.
        self.fuse_loss = bool(fuse_loss) and self.L >= 2 and self.xform_first[-1]
        self.keep_logits = keep_logits
        self.P_last = mat(dims[-1], act) if self.fuse_loss else None
        self.dW = [torch.empty_like(w) for w, _ in weights]
        self._dW0 = None
        if self.d_in_padded != dims[0]:
            self._dW0 = torch.zeros_like(self._W0)
            self.dW[0] = self._dW0[:dims[0]]
        self.db = [torch.empty_like(b) for _, b in weights]
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)

    def _new_batch(self):
        """Device buffers of one mini-batch: the sample, its bitmap and rank prefix, the induced CSR
        (with its long-row plan), the sliced labels and (unfused) features."""
        W = (self.N + 63) // 64
        dev = self.dev
        b = type("Batch", (), {})()
        b.S = torch.empty(self.B, dtype=torch.int32, device=dev)
        b.bitmap = torch.empty(W, dtype=torch.int64, device=dev)
        b.rank = torch.empty(W, dtype=torch.int32, device=dev)
        b.A = sg.Csr(self.B, self.B, self.capacity, dev)
        b.y_S = torch.empty(self.B, dtype=torch.int32, device=dev)
        b.X_S = None if self.fuse_slice else torch.empty((self.B, self.dims[0]), dtype=torch.float32, device=dev)
        b.ready = torch.cuda.Event()
        b.free = torch.cuda.Event()
        return b

    def _use(self, b):
        self.S, self.bitmap, self.rank, self.A, self.y_S, self.X_S = b.S, b.bitmap, b.rank, b.A, b.y_S, b.X_S

    def sample(self, t: int):
        sg.sgnn_sample_uniform(self.ctx, self.N, self.B, self.seed, t, self.S, self.bitmap, self.rank)

    def induce(self):
        sg.sgnn_induced_csr(self.ctx, self.N, self.rowptr, self.colidx, None, self.S, self.B, self.bitmap, self.rank,
                            self.A)

    def slice(self):
        sg.sgnn_gather_rows(self.ctx, None if self.fuse_slice else self.X, self.S, self.B, self.X_S, self.labels,
                            self.y_S)

    def forward(self, after_first=None):
        """after_first: called once the first layer has been issued (the captured pipeline forks there)."""
        for l, (W, b) in enumerate(self.weights):
            flags = self.flags | (sg.SGNN_RELU if l < self.L - 1 else 0) | (sg.SGNN_XFORM_FIRST if self.xform_first[l] else 0)
            if l == self.L - 1 and self.fuse_loss:
                sg.sgnn_gemm(self.ctx, False, False, self.H[l - 1], W, None, self.flags, self.P_last)   # the rest with the loss
                continue
            if l == 0 and self.fuse_slice:
                if self._dW0 is not None:
                    W = self._W0
                sg.sgnn_gcn_fwd(self.ctx, self.A, self.X, W, b, flags, self.H[0], self.T[0], row_index=self.S)
            else:
                Hin = self.X_S if l == 0 else self.H[l - 1]
                sg.sgnn_gcn_fwd(self.ctx, self.A, Hin, W, b, flags, self.H[l], self.T[l])
            if l == 0 and after_first is not None:
                after_first()

    def loss_and_grad(self):
        # the last layer has no activation: its bias gradient is the column sum of dO, taken in the same pass
        if self.fuse_loss:
            sg.sgnn_spmm_xent(self.ctx, self.A, self.P_last, self.weights[-1][1], self.y_S, self.loss, self.dO,
                              O=self.H[-1] if self.keep_logits else None, dO_colsum=self.db[-1])
            return
        sg.sgnn_softmax_xent(self.ctx, self.H[-1], self.y_S, self.loss, self.dO, dO_colsum=self.db[-1])

    def backward(self, side=None, before_last=None):
        """side = (stream, context): the weight gradients dW = T^T dZ of the layers whose dZ is the incoming
        dY itself (no masking pass in between) are computed there, concurrently with the rest of the backward
        pass on the current stream; the caller joins the two streams.
        before_last: called before the first layer's backward is issued (the captured pipeline joins there)."""
        dY = self.dO
        masked = False    # dY already carries the ReLU mask of the layer it enters
        for l in range(self.L - 1, -1, -1):
            W, _ = self.weights[l]
            relu = l < self.L - 1
            flags = self.flags | (sg.SGNN_RELU if relu else 0) | (sg.SGNN_XFORM_FIRST if self.xform_first[l] else 0)
            if masked:
                flags |= sg.SGNN_DY_MASKED
            saved, ridx = self.T[l], None
            if self.xform_first[l]:
                if l == 0:
                    saved, ridx = (self.X, self.S) if self.fuse_slice else (self.X_S, None)
                else:
                    saved = self.H[l - 1]
            dW, db = self.dW[l], self.db[l]
            if l == 0 and self._dW0 is not None:
                W, dW = self._W0, self._dW0
            if l == self.L - 1:
                db = None                            # came with the loss gradient
            if l == 0 and before_last is not None:
                before_last()
            if side is not None and not self.xform_first[l] and (masked or not relu):
                main = torch.cuda.current_stream()
                ev = torch.cuda.Event()
                ev.record(main)                      # dY is complete
                side[0].wait_event(ev)
                sg.sgnn_gemm(side[1], True, False, saved, dY, None, self.flags, dW, stream=side[0], b_colsum=db)
                dW = db = None
            # the ReLU backward of the layer below is fused into the product that writes dH
            fuse = self.fuse_relu_bwd and l > 0
            # the induced matrix of a symmetric graph is symmetric: it is its own transpose
            sg.sgnn_gcn_bwd(self.ctx, self.A, saved, W, self.H[l], dY, flags, self.dH[l], dW, db,
                            row_index=ridx, H_in=self.H[l - 1] if fuse else None)
            dY = self.dH[l]
            masked = fuse

    def step(self, t: int):
        """One whole step on the current stream."""
        self.sample(t)
        self.induce()
        self.slice()
        self.forward()
        self.loss_and_grad()
        self.backward()

    # ---- sampling of step t+1 overlapped with the training of step t (Sec. V-A of the paper) ----

    def _build(self, t: int, b, ctx, st):
        """sample -> induced CSR -> slice for step t into batch b, on stream st with the context ctx."""
        sg.sgnn_sample_uniform(ctx, self.N, self.B, self.seed, t, b.S, b.bitmap, b.rank, stream=st)
        sg.sgnn_induced_csr(ctx, self.N, self.rowptr, self.colidx, None, b.S, self.B, b.bitmap, b.rank, b.A, stream=st)
        sg.sgnn_gather_rows(ctx, None if self.fuse_slice else self.X, b.S, self.B, b.X_S, self.labels, b.y_S, stream=st)

    def _prefetch(self, t: int, b, wait_free: bool = True):
        """The mini-batch of step t built into batch b on the side stream with its own context (scratch),
        after the training that last used b has finished."""
        st = self.side_stream
        if wait_free:
            st.wait_event(b.free)
        self._build(t, b, self.side_ctx, st)
        b.ready.record(st)

    def _init_side(self):
        if not hasattr(self, "side_stream"):
            self.side_stream = torch.cuda.Stream(device=self.dev)       # default priority
            self.side_ctx = sg.Context(self.dev.index or 0)
            self.side_ctx.reserve(self.N, int(self.colidx.numel()), self.B, max(self.dims), self.capacity)
            self.batches.append(self._new_batch())
            main = torch.cuda.current_stream()
            for b in self.batches:
                b.free.record(main)

    def run(self, steps):
        """Run the given steps with the mini-batch of the next step built on a second stream while
        the current one trains.  The prefetch crosses whatever boundary (epoch) the list contains.
        Results of the last step are left in the usual buffers; returns nothing."""
        steps = list(steps)
        if not steps:
            return
        self._init_side()
        main = torch.cuda.current_stream()
        self.side_stream.wait_stream(main)       # earlier work on the main stream that wrote the buffers
        self._prefetch(steps[0], self.batches[0])
        for i, t in enumerate(steps):
            b = self.batches[i % 2]
            if i + 1 < len(steps):
                self._prefetch(steps[i + 1], self.batches[(i + 1) % 2])
            main.wait_event(b.ready)
            self._use(b)
            self.forward()
            self.loss_and_grad()
            self.backward(side=(self.side_stream, self.side_ctx) if self.side_dw else None)
            if self.side_dw:
                main.wait_stream(self.side_stream)     # the weight gradients computed over there
            b.free.record(main)
        main.wait_stream(self.side_stream)

    # ---- the same pipeline captured in HIP graphs (one per mini-batch of a cycle) ----

    def build_graphs(self, cycle, steps_per_graph: int = 0, fork: str = "mid"):
        """Capture the overlapped pipeline over a cycle of steps (even length) in HIP graphs of
        steps_per_graph steps each (0 = the whole cycle in one graph; must be even and divide the cycle).
        Every step trains the mini-batch of cycle[i] (already in buffer set i % 2) while it builds the
        one of cycle[i+1] in the other set on a forked stream.  Replaying the graphs in order, round and
        round, is the overlapped pipeline without any per-kernel launch work on the host.

        fork = "mid": the builder leaves the main stream after the step's first layer and rejoins it before
        its last backward call, so the kernels on either side of a step boundary follow each other without
        a dependency on another queue (a few percent faster than "start", where the builder is forked at the
        start of the step and joined at its end)."""
        cycle = list(cycle)
        spg = steps_per_graph or len(cycle)
        if len(cycle) % 2 or spg % 2 or len(cycle) % spg:
            raise ValueError("the cycle and the steps per graph must be even, and the latter must divide the former")
        if fork not in ("mid", "start"):
            raise ValueError("fork must be 'mid' or 'start'")
        self._init_side()
        torch.cuda.synchronize()
        self.cycle, self.graphs, self.steps_per_graph = cycle, [], spg
        cap = torch.cuda.Stream(device=self.dev)
        for g0 in range(0, len(cycle), spg):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=cap):
                main = torch.cuda.current_stream()
                for i in range(g0, g0 + spg):
                    b, nb = self.batches[i % 2], self.batches[(i + 1) % 2]

                    def fork_prefetch(t=cycle[(i + 1) % len(cycle)], nb=nb):
                        self.side_stream.wait_stream(main)
                        self._prefetch(t, nb, wait_free=False)

                    def join():
                        main.wait_stream(self.side_stream)

                    side = (self.side_stream, self.side_ctx) if self.side_dw else None
                    self._use(b)
                    if fork == "mid":
                        self.forward(after_first=fork_prefetch)
                        self.loss_and_grad()
                        self.backward(side=side, before_last=join)
                        if self.side_dw:
                            join()
                    else:
                        fork_prefetch()
                        self.forward()
                        self.loss_and_grad()
                        self.backward(side=side)
                        join()
            self.graphs.append(g)
        torch.cuda.synchronize()

    def run_graphs(self, n: int):
        """n steps of the captured cycle, starting at its first step (n a multiple of the steps per graph)."""
        if n % self.steps_per_graph:
            raise ValueError("n must be a multiple of the %d steps of a graph" % self.steps_per_graph)
        self.side_stream.wait_stream(torch.cuda.current_stream())
        self._prefetch(self.cycle[0], self.batches[0], wait_free=False)
        torch.cuda.current_stream().wait_stream(self.side_stream)
        for i in range(n // self.steps_per_graph):
            self.graphs[i % len(self.graphs)].replay()
        self._use(self.batches[(n - 1) % 2])
