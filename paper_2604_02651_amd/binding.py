"""ctypes binding of libsgnn.so: the same entry points as include/sgnn.h, taking torch tensors.

Argument marshalling only.  Tensors must live on the context's GPU, be contiguous in their last
dimension and have the dtype the C declaration states; the functions check that, pass raw device
pointers, and raise SgnnError with the library's message on a negative return code.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("SGNN_LIB_PATH") or os.path.join(_HERE, "libsgnn.so")   # the override is for trying out builds

SGNN_RELU = 1
SGNN_BF16_MFMA = 2
SGNN_XFORM_FIRST = 4
SGNN_DY_MASKED = 8
SGNN_FUSE_TAIL = 16
SGNN_F32 = 0
SGNN_BF16 = 1

_ERR_NAMES = {-1: "SGNN_ERR_INVALID_ARG", -2: "SGNN_ERR_CAPACITY", -3: "SGNN_ERR_UNSUPPORTED", -4: "SGNN_ERR_HIP",
              -5: "SGNN_ERR_INTERNAL"}


class SgnnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("%s (%d): %s" % (_ERR_NAMES.get(code, "SGNN_ERR"), code, message))
        self.code = code


class _Graph(C.Structure):
    _fields_ = [("N", C.c_uint64), ("E", C.c_uint64), ("rowptr", C.c_void_p), ("rowptr_is_i64", C.c_int),
                ("colidx", C.c_void_p), ("val", C.c_void_p)]


class _Csr(C.Structure):
    _fields_ = [("rows", C.c_uint32), ("cols", C.c_uint32), ("rowptr", C.c_void_p), ("colidx", C.c_void_p),
                ("val", C.c_void_p), ("capacity", C.c_uint64), ("nnz_dev", C.c_void_p), ("plan", C.c_void_p),
                ("rowptr_is_i64", C.c_int)]


class _Mat(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("row_index", C.c_void_p)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded C library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libsgnn.so is not built: run `python -m paper_2604_02651_amd.build` "
                              "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = C.CDLL(_LIB_PATH)
        vp, u64, u32, i64, ci = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int64, C.c_int
        L.sgnn_ctx_create.argtypes = [C.POINTER(vp), ci]
        L.sgnn_ctx_destroy.argtypes = [vp]
        L.sgnn_ctx_reserve.argtypes = [vp, u64, u64, u32, u32, u64]
        L.sgnn_last_error.argtypes = [vp]
        L.sgnn_last_error.restype = C.c_char_p
        L.sgnn_ctx_status.argtypes = [vp, vp]
        L.sgnn_ctx_profile.argtypes = [vp, ci]
        L.sgnn_ctx_profile_read.argtypes = [vp, C.c_char_p, u64]
        L.sgnn_sample_uniform.argtypes = [vp, u64, u32, u64, u64, vp, vp, vp, vp]
        L.sgnn_sample_uniform_static.argtypes = [u64, u32, u64, u64, vp, vp, vp, vp, vp]
        L.sgnn_induced_csr.argtypes = [vp, C.POINTER(_Graph), vp, u32, vp, vp, ci, ci, C.POINTER(_Csr),
                                       C.POINTER(u64), vp]
        L.sgnn_csr_plan_bytes.argtypes = [u32, u64]
        L.sgnn_csr_plan_bytes.restype = u64
        L.sgnn_csr_plan.argtypes = [vp, C.POINTER(_Csr), vp]
        L.sgnn_gather_rows.argtypes = [vp, vp, i64, i64, vp, u32, vp, i64, vp, vp, vp]
        L.sgnn_gcn_fwd.argtypes = [vp, C.POINTER(_Csr), C.POINTER(_Mat), C.POINTER(_Mat), vp, ci, C.POINTER(_Mat),
                                   C.POINTER(_Mat), vp]
        L.sgnn_gcn_bwd.argtypes = [vp, C.POINTER(_Csr), C.POINTER(_Mat), C.POINTER(_Mat), C.POINTER(_Mat),
                                   C.POINTER(_Mat), ci, C.POINTER(_Mat), C.POINTER(_Mat), vp, vp, vp]
        u64, cf = C.c_uint64, C.c_float
        L.sgnn_tail_fwd.argtypes = [vp, C.POINTER(_Mat), vp, cf, C.POINTER(_Mat), cf, u64, u32, u64, C.POINTER(_Mat), vp, vp]
        L.sgnn_gemm_tail_fwd.argtypes = [vp, C.POINTER(_Mat), C.POINTER(_Mat), vp, cf, C.POINTER(_Mat), cf, u64, u32, u64, ci,
                                         C.POINTER(_Mat), C.POINTER(_Mat), vp, vp]
        L.sgnn_tail_bwd.argtypes = [vp, C.POINTER(_Mat), vp, vp, cf, u64, u32, u64, C.POINTER(_Mat), C.POINTER(_Mat), vp, vp,
                                    vp]
        cd = C.c_double
        L.sgnn_sgd_step.argtypes = [vp, vp, vp, i64, cd, cd, vp]
        L.sgnn_adam_step.argtypes = [vp, vp, vp, vp, vp, i64, cd, cd, cd, cd, i64, vp]
        L.sgnn_graph_normalized_csr.argtypes = [vp, C.POINTER(_Graph), vp, vp, vp]
        L.sgnn_induced_csr_range.argtypes = [vp, C.POINTER(_Graph), vp, u32, vp, vp, ci, i64, i64, i64, i64, C.POINTER(_Csr), vp, vp]
        L.sgnn_csr_transpose.argtypes = [vp, C.POINTER(_Csr), C.POINTER(_Csr), vp]
        L.sgnn_sigmoid_bce.argtypes = [vp, vp, i64, vp, i64, u32, u32, vp, vp, i64, vp]
        L.sgnn_colsum.argtypes = [vp, C.POINTER(_Mat), vp, vp]
        L.sgnn_softmax_xent.argtypes = [vp, vp, i64, vp, u32, u32, vp, vp, C.c_int, i64, vp, vp]
        L.sgnn_spmm_xent.argtypes = [vp, C.POINTER(_Csr), C.POINTER(_Mat), vp, vp, C.POINTER(_Mat), vp, vp, C.c_int, i64, vp, vp]
        L.sgnn_spmm.argtypes = [vp, C.POINTER(_Csr), C.POINTER(_Mat), C.POINTER(_Mat), C.POINTER(_Mat), vp]
        L.sgnn_copy_f32.argtypes = [vp, vp, vp, i64, vp]
        L.sgnn_gemm.argtypes = [vp, ci, ci, i64, i64, i64, vp, ci, i64, vp, ci, i64, vp, ci, vp, ci, i64, vp, ci, i64, vp, vp]
        for name in ("sgnn_ctx_create", "sgnn_ctx_destroy", "sgnn_ctx_reserve", "sgnn_ctx_status",
                     "sgnn_ctx_profile", "sgnn_ctx_profile_read",
                     "sgnn_sample_uniform", "sgnn_induced_csr", "sgnn_csr_plan", "sgnn_gather_rows", "sgnn_gcn_fwd", "sgnn_gcn_bwd", "sgnn_tail_fwd", "sgnn_tail_bwd", "sgnn_gemm_tail_fwd", "sgnn_sgd_step", "sgnn_adam_step", "sgnn_graph_normalized_csr", "sgnn_induced_csr_range", "sgnn_csr_transpose", "sgnn_sigmoid_bce", "sgnn_colsum",
                     "sgnn_softmax_xent", "sgnn_spmm_xent", "sgnn_spmm", "sgnn_gemm", "sgnn_copy_f32"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return C.c_void_p(h)


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("%s must be a CUDA/HIP tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if t.dim() >= 1 and t.numel() > 0 and t.stride(-1) != 1:
        raise TypeError("%s must be contiguous in its last dimension" % name)
    return C.c_void_p(t.data_ptr())


def _mat(t: torch.Tensor, row_index: Optional[torch.Tensor] = None, name="matrix", allow_bf16: bool = False) -> _Mat:
    """allow_bf16: the matrix may be stored as bfloat16 (the input operand of a sparse product)."""
    if t.dim() != 2:
        raise TypeError("%s must be 2-D" % name)
    bf16 = allow_bf16 and t.dtype == torch.bfloat16
    p = _ptr(t, torch.bfloat16 if bf16 else torch.float32, name)
    ri = _ptr(row_index, torch.int32, name + ".row_index")
    rows = row_index.numel() if row_index is not None else t.shape[0]
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return _Mat(p, SGNN_BF16 if bf16 else SGNN_F32, rows, t.shape[1], ld, ri)


class Context:
    """Owns an sgnn_ctx.  One context per concurrently used stream."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        self.device = device
        rc = lib().sgnn_ctx_create(C.byref(self._h), device)
        if rc != 0:
            raise SgnnError(rc, "sgnn_ctx_create failed (is a GPU visible?)")

    def check(self, rc: int):
        if rc != 0:
            raise SgnnError(rc, lib().sgnn_last_error(self._h).decode())

    def reserve(self, N: int, E: int, B: int, d_max: int, max_entries: int = 0):
        self.check(lib().sgnn_ctx_reserve(self._h, N, E, B, d_max, max_entries))

    def status(self, stream=None):
        self.check(lib().sgnn_ctx_status(self._h, _stream(stream)))

    def profile(self, enable: bool):
        self.check(lib().sgnn_ctx_profile(self._h, int(enable)))

    def profile_read(self):
        """[(kernel, tag, launches, total_ms)] recorded since profiling was enabled."""
        buf = C.create_string_buffer(1 << 20)
        self.check(lib().sgnn_ctx_profile_read(self._h, buf, len(buf)))
        out = []
        for line in buf.value.decode().splitlines():
            name, tag, calls, ms = line.split("\t")
            out.append((name, tag, int(calls), float(ms)))
        return out

    def close(self):
        if self._h:
            lib().sgnn_ctx_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Csr:
    """Device buffers of a mini-batch CSR (rows x cols) with room for `capacity` entries."""

    def __init__(self, rows: int, cols: int, capacity: int, device="cuda:0", with_plan: bool = True):
        self.rows, self.cols, self.capacity = rows, cols, capacity
        self.plan = None
        if with_plan:
            nbytes = int(lib().sgnn_csr_plan_bytes(rows, capacity))
            self.plan = torch.zeros((nbytes + 7) // 8, dtype=torch.int64, device=device)
        self.rowptr = torch.zeros(rows + 1, dtype=torch.int32, device=device)
        self.colidx = torch.zeros(max(capacity, 1), dtype=torch.int32, device=device)
        self.val = torch.zeros(max(capacity, 1), dtype=torch.float32, device=device)
        self.nnz_dev = torch.zeros(1, dtype=torch.int32, device=device)

    @classmethod
    def from_arrays(cls, rows, cols, rowptr, colidx, val, device="cuda:0", with_plan: bool = False):
        """A matrix from host arrays.  Without with_plan the sparse products plan on the fly; with
        it, call sgnn_csr_plan(ctx, csr) once after this."""
        import numpy as np
        c = cls(rows, cols, len(colidx), device, with_plan)
        c.rowptr.copy_(torch.as_tensor(np.asarray(rowptr, np.int32)))
        if len(colidx):
            c.colidx[:len(colidx)].copy_(torch.as_tensor(np.asarray(colidx, np.int32)))
            c.val[:len(colidx)].copy_(torch.as_tensor(np.asarray(val, np.float32)))
        c.nnz_dev.fill_(len(colidx))
        return c

    def struct(self) -> _Csr:
        i64 = self.rowptr.dtype == torch.int64         # a full graph with 2^31 entries or more (sparse products only)
        return _Csr(self.rows, self.cols, _ptr(self.rowptr, torch.int64 if i64 else torch.int32), _ptr(self.colidx, torch.int32),
                    _ptr(self.val, torch.float32), self.capacity, _ptr(self.nnz_dev, torch.int32),
                    _ptr(self.plan, torch.int64) if self.plan is not None else None, int(i64))

    def nnz(self) -> int:
        return int(self.nnz_dev.item()) if self.nnz_dev is not None else int(self.rowptr[-1].item())


# ------------------------------------------------------------------------------------------------
# entry points, named as in include/sgnn.h
# ------------------------------------------------------------------------------------------------

def sgnn_sample_uniform(ctx: Context, N: int, B: int, seed: int, step: int, S: torch.Tensor, bitmap: torch.Tensor,
                        rank: torch.Tensor, stream=None):
    """S int32[B], bitmap int64[ceil(N/64)] (the bits of the C uint64 words), rank int32[ceil(N/64)]."""
    W = (N + 63) // 64
    if S is not None and S.numel() < B or bitmap is not None and bitmap.numel() < W or rank is not None and rank.numel() < W:
        raise ValueError("output tensor too small")
    ctx.check(lib().sgnn_sample_uniform(ctx._h, N, B, seed & (2**64 - 1), step & (2**64 - 1), _ptr(S, torch.int32, "S"),
                                        _ptr(bitmap, torch.int64, "bitmap"), _ptr(rank, torch.int32, "rank"),
                                        _stream(stream)))


def sgnn_sample_uniform_static(N: int, B: int, seed: int, step: int, S: torch.Tensor, bitmap: torch.Tensor,
                               rank: torch.Tensor, status: Optional[torch.Tensor] = None, stream=None):
    """sgnn_sample_uniform without a context and without any allocation, on the current device of S."""
    W = (N + 63) // 64
    if S.numel() < B or bitmap.numel() < W or rank.numel() < W:
        raise ValueError("output tensor too small")
    with torch.cuda.device(S.device):
        rc = lib().sgnn_sample_uniform_static(N, B, seed & (2**64 - 1), step & (2**64 - 1), _ptr(S, torch.int32, "S"),
                                              _ptr(bitmap, torch.int64, "bitmap"), _ptr(rank, torch.int32, "rank"),
                                              _ptr(status, torch.int32, "status"), _stream(stream))
    if rc < 0:
        raise SgnnError(rc, lib().sgnn_last_error(None).decode())


def sgnn_induced_csr(ctx: Context, N: int, rowptr: torch.Tensor, colidx: torch.Tensor, val: Optional[torch.Tensor],
                     S: torch.Tensor, B: int, bitmap: torch.Tensor, rank: torch.Tensor, out: Csr,
                     norm_mode: int = 0, rescale: int = 1, want_nnz: bool = False, stream=None) -> Optional[int]:
    """Returns the entry count when want_nnz (synchronises), else None."""
    if rowptr.dtype not in (torch.int32, torch.int64):
        raise TypeError("rowptr must be int32 or int64")
    if rowptr.numel() != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    g = _Graph(N, colidx.numel(), _ptr(rowptr, None, "rowptr"), int(rowptr.dtype == torch.int64),
               _ptr(colidx, torch.int32, "colidx"), _ptr(val, torch.float32, "val"))
    if out.rowptr.numel() < B + 1:
        raise ValueError("out.rowptr too small")
    cs = out.struct()
    nnz = C.c_uint64(0)
    rc = lib().sgnn_induced_csr(ctx._h, C.byref(g), _ptr(S, torch.int32, "S"), B, _ptr(bitmap, torch.int64, "bitmap"),
                                _ptr(rank, torch.int32, "rank"), norm_mode, rescale, C.byref(cs),
                                C.byref(nnz) if want_nnz else None, _stream(stream))
    out.rows = out.cols = B
    ctx.check(rc)
    return int(nnz.value) if want_nnz else None


def sgnn_graph_normalized_csr(ctx: Context, N: int, rowptr: torch.Tensor, colidx: torch.Tensor,
                              val: Optional[torch.Tensor] = None, with_plan: bool = True, stream=None) -> Csr:
    """The full graph as an N x N Csr for the full-graph evaluation forward: int32 row offsets and the weights of
    Eq. 3 are written by the library; the column indices are the graph's own tensor (shared, not copied)."""
    if rowptr.numel() != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    E = int(colidx.numel())
    g = _Graph(N, E, _ptr(rowptr, None, "rowptr"), int(rowptr.dtype == torch.int64), _ptr(colidx, torch.int32, "colidx"),
               _ptr(val, torch.float32, "val"))
    out = Csr.__new__(Csr)
    out.rows, out.cols, out.capacity = N, N, E
    dev = colidx.device
    big = E >= 2 ** 31 - 1
    out.rowptr = rowptr if big else torch.empty(N + 1, dtype=torch.int32, device=dev)     # the graph's own int64 offsets when 32 bits do not do
    out.colidx = colidx
    out.val = torch.empty(max(E, 1), dtype=torch.float32, device=dev)
    out.nnz_dev = None if big else torch.full((1,), E, dtype=torch.int32, device=dev)
    out.plan = None
    ctx.check(lib().sgnn_graph_normalized_csr(ctx._h, C.byref(g), None if big else _ptr(out.rowptr, torch.int32),
                                              _ptr(out.val, torch.float32), _stream(stream)))
    if with_plan:
        nbytes = int(lib().sgnn_csr_plan_bytes(N, E))
        out.plan = torch.zeros((nbytes + 7) // 8, dtype=torch.int64, device=dev)
        sgnn_csr_plan(ctx, out, stream=stream)
    return out


def sgnn_induced_csr_range(ctx: Context, N: int, rowptr: torch.Tensor, colidx: torch.Tensor, val: Optional[torch.Tensor],
                           S: torch.Tensor, B: int, bitmap: torch.Tensor, rank: torch.Tensor, R0: int, R1: int, C0: int,
                           C1: int, out: Csr, rescale: int = 1, want_nnz: bool = False, stream=None) -> Optional[int]:
    """One shard (rows of S in [R0, R1), columns of S in [C0, C1)) of the mini-batch matrix; B x B namespace."""
    if rowptr.numel() != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    g = _Graph(N, colidx.numel(), _ptr(rowptr, None, "rowptr"), int(rowptr.dtype == torch.int64),
               _ptr(colidx, torch.int32, "colidx"), _ptr(val, torch.float32, "val"))
    cs = out.struct()
    nnz = C.c_uint64(0)
    rc = lib().sgnn_induced_csr_range(ctx._h, C.byref(g), _ptr(S, torch.int32, "S"), B, _ptr(bitmap, torch.int64, "bitmap"),
                                      _ptr(rank, torch.int32, "rank"), rescale, R0, R1, C0, C1, C.byref(cs),
                                      C.byref(nnz) if want_nnz else None, _stream(stream))
    out.rows = out.cols = B
    ctx.check(rc)
    return int(nnz.value) if want_nnz else None


def sgnn_csr_transpose(ctx: Context, A: Csr, out: Csr, stream=None):
    """out = A^T (out: cols x rows of A, capacity >= A's)."""
    a, o = A.struct(), out.struct()
    ctx.check(lib().sgnn_csr_transpose(ctx._h, C.byref(a), C.byref(o), _stream(stream)))


def sgnn_csr_plan(ctx: Context, A: Csr, stream=None):
    a = A.struct()
    ctx.check(lib().sgnn_csr_plan(ctx._h, C.byref(a), _stream(stream)))


def sgnn_gather_rows(ctx: Context, X: Optional[torch.Tensor], S: torch.Tensor, B: int, out: Optional[torch.Tensor],
                     labels: Optional[torch.Tensor] = None, labels_out: Optional[torch.Tensor] = None, stream=None):
    if X is not None and (out.shape[0] < B or out.shape[1] != X.shape[1]):
        raise ValueError("out has the wrong shape")
    d, ldx, ldo = (X.shape[1], X.stride(0), out.stride(0)) if X is not None else (0, 0, 0)
    ctx.check(lib().sgnn_gather_rows(ctx._h, _ptr(X, torch.float32, "X"), d, ldx,
                                     _ptr(S, torch.int32, "S"), B, _ptr(out, torch.float32, "out"), ldo,
                                     _ptr(labels, torch.int32, "labels"), _ptr(labels_out, torch.int32, "labels_out"),
                                     _stream(stream)))


def sgnn_gcn_fwd(ctx: Context, A: Csr, H: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor], flags: int,
                 Y: torch.Tensor, T: Optional[torch.Tensor], row_index: Optional[torch.Tensor] = None, stream=None):
    a = A.struct()
    h, w, y = _mat(H, row_index, "H", allow_bf16=True), _mat(W, None, "W"), _mat(Y, None, "Y", allow_bf16=True)
    t = _mat(T, None, "T", allow_bf16=True) if T is not None else None
    ctx.check(lib().sgnn_gcn_fwd(ctx._h, C.byref(a), C.byref(h), C.byref(w), _ptr(bias, torch.float32, "bias"), flags,
                                 C.byref(y), C.byref(t) if t is not None else None, _stream(stream)))


def sgnn_gcn_bwd(ctx: Context, A_T: Csr, T: torch.Tensor, W: torch.Tensor, Y: Optional[torch.Tensor], dY: torch.Tensor,
                 flags: int, dH: Optional[torch.Tensor], dW: Optional[torch.Tensor], dbias: Optional[torch.Tensor],
                 row_index: Optional[torch.Tensor] = None, stream=None, H_in: Optional[torch.Tensor] = None):
    """T is the saved aggregate, or with SGNN_XFORM_FIRST the layer input (row_index honoured).
    H_in (the layer input, output of the ReLU below): dH comes back multiplied by [H_in > 0]."""
    a = A_T.struct()
    t, w, dy = _mat(T, row_index, "T", allow_bf16=True), _mat(W, None, "W"), _mat(dY, None, "dY", allow_bf16=True)
    y = _mat(Y, None, "Y", allow_bf16=True) if Y is not None else None
    dh = _mat(dH, None, "dH", allow_bf16=True) if dH is not None else None
    hin = _mat(H_in, None, "H_in", allow_bf16=True) if H_in is not None else None
    if dW is not None and (dW.shape != W.shape or not dW.is_contiguous()):
        raise ValueError("dW must be contiguous with the shape of W")
    ctx.check(lib().sgnn_gcn_bwd(ctx._h, C.byref(a), C.byref(t), C.byref(w), C.byref(y) if y is not None else None,
                                 C.byref(dy), flags, C.byref(dh) if dh is not None else None,
                                 C.byref(hin) if hin is not None else None, _ptr(dW, torch.float32, "dW"), _ptr(dbias, torch.float32, "dbias"), _stream(stream)))


def sgnn_sigmoid_bce(ctx: Context, O: torch.Tensor, Y: torch.Tensor, loss: Optional[torch.Tensor],
                     dO: Optional[torch.Tensor], stream=None):
    """Mean binary cross-entropy on logits (multi-label loss) and its gradient."""
    ctx.check(lib().sgnn_sigmoid_bce(ctx._h, _ptr(O, torch.float32, "O"), O.stride(0), _ptr(Y, torch.float32, "Y"), Y.stride(0),
                                     O.shape[0], O.shape[1], _ptr(loss, torch.float32, "loss"), _ptr(dO, torch.float32, "dO"),
                                     dO.stride(0) if dO is not None else 0, _stream(stream)))


def sgnn_colsum(ctx: Context, X: torch.Tensor, out: torch.Tensor, stream=None):
    """out[j] = sum_i X[i, j] (fixed order)."""
    x = _mat(X, None, "X")
    ctx.check(lib().sgnn_colsum(ctx._h, C.byref(x), _ptr(out, torch.float32, "out"), _stream(stream)))


def sgnn_tail_fwd(ctx: Context, Z: torch.Tensor, gamma: Optional[torch.Tensor], eps: float, R: Optional[torch.Tensor],
                  drop_q: float, drop_seed: int, layer: int, step: int, Y: torch.Tensor, inv_rms: Optional[torch.Tensor],
                  stream=None):
    """Y = dropout(relu(rmsnorm(Z; gamma, eps)), drop_q) + R; inv_rms (fp32[B]) is kept for sgnn_tail_bwd."""
    z, y = _mat(Z, None, "Z"), _mat(Y, None, "Y")
    r = _mat(R, None, "R") if R is not None else None
    ctx.check(lib().sgnn_tail_fwd(ctx._h, C.byref(z), _ptr(gamma, torch.float32, "gamma"), eps,
                                  C.byref(r) if r is not None else None, drop_q, drop_seed, layer, step, C.byref(y),
                                  _ptr(inv_rms, torch.float32, "inv_rms"), _stream(stream)))


def sgnn_gemm_tail_fwd(ctx: Context, T: torch.Tensor, W: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                       R: Optional[torch.Tensor], drop_q: float, drop_seed: int, layer: int, step: int, flags: int,
                       Z: torch.Tensor, Y: torch.Tensor, inv_rms: Optional[torch.Tensor], stream=None):
    """Z = T W and Y = dropout(relu(rmsnorm(Z))) + R in one call (one kernel for tall bf16 products)."""
    t, w, z, y = _mat(T, None, "T"), _mat(W, None, "W"), _mat(Z, None, "Z"), _mat(Y, None, "Y")
    r = _mat(R, None, "R") if R is not None else None
    ctx.check(lib().sgnn_gemm_tail_fwd(ctx._h, C.byref(t), C.byref(w), _ptr(gamma, torch.float32, "gamma"), eps,
                                       C.byref(r) if r is not None else None, drop_q, drop_seed, layer, step, flags,
                                       C.byref(z), C.byref(y), _ptr(inv_rms, torch.float32, "inv_rms"), _stream(stream)))


def sgnn_tail_bwd(ctx: Context, Z: torch.Tensor, inv_rms: torch.Tensor, gamma: Optional[torch.Tensor], drop_q: float,
                  drop_seed: int, layer: int, step: int, dY: torch.Tensor, dZ: torch.Tensor,
                  dgamma: Optional[torch.Tensor], dbias: Optional[torch.Tensor], stream=None):
    z, dy, dz = _mat(Z, None, "Z"), _mat(dY, None, "dY"), _mat(dZ, None, "dZ")
    ctx.check(lib().sgnn_tail_bwd(ctx._h, C.byref(z), _ptr(inv_rms, torch.float32, "inv_rms"),
                                  _ptr(gamma, torch.float32, "gamma"), drop_q, drop_seed, layer, step, C.byref(dy), C.byref(dz),
                                  _ptr(dgamma, torch.float32, "dgamma"), _ptr(dbias, torch.float32, "dbias"), _stream(stream)))


def sgnn_softmax_xent(ctx: Context, O: torch.Tensor, labels: torch.Tensor, loss: Optional[torch.Tensor],
                      dO: Optional[torch.Tensor], stream=None, dO_colsum: Optional[torch.Tensor] = None):
    """dO_colsum: optional float[C], receives the column sums of dO (the bias gradient of a last layer without activation)."""
    if dO_colsum is not None and dO_colsum.numel() != O.shape[1]:
        raise ValueError("dO_colsum must have one element per class")
    if dO is not None and (dO.shape != O.shape or dO.stride(1) != 1):
        raise ValueError("dO must have the shape of O and unit column stride")
    ctx.check(lib().sgnn_softmax_xent(ctx._h, _ptr(O, torch.float32, "O"), O.stride(0), _ptr(labels, torch.int32, "labels"),
                                      O.shape[0], O.shape[1], _ptr(loss, torch.float32, "loss"),
                                      _ptr(dO, dO.dtype if dO is not None and dO.dtype == torch.bfloat16 else torch.float32, "dO"),
                                      _dt(dO, "dO"), dO.stride(0) if dO is not None else 0,
                                      _ptr(dO_colsum, torch.float32, "dO_colsum"), _stream(stream)))


def sgnn_spmm_xent(ctx: Context, A: Csr, X: torch.Tensor, bias: Optional[torch.Tensor], labels: torch.Tensor,
                   loss: Optional[torch.Tensor], dO: Optional[torch.Tensor], O: Optional[torch.Tensor] = None,
                   dO_colsum: Optional[torch.Tensor] = None, stream=None):
    """O = A X + bias, its mean softmax cross-entropy against labels and the gradient dO, in one pass.  O None: the
    logits are not kept."""
    a = A.struct()
    x = _mat(X, None, "X", allow_bf16=True)
    o = _mat(O, None, "O") if O is not None else None
    if bias is not None and bias.numel() != X.shape[1]:
        raise ValueError("bias must have one element per class")
    if dO is not None and (tuple(dO.shape) != (A.rows, X.shape[1]) or dO.stride(1) != 1):
        raise ValueError("dO must be rows x classes with unit column stride")
    if dO_colsum is not None and dO_colsum.numel() != X.shape[1]:
        raise ValueError("dO_colsum must have one element per class")
    if labels.numel() != A.rows:
        raise ValueError("one label per row")
    ctx.check(lib().sgnn_spmm_xent(ctx._h, C.byref(a), C.byref(x), _ptr(bias, torch.float32, "bias"), _ptr(labels, torch.int32, "labels"),
                                   C.byref(o) if o is not None else None, _ptr(loss, torch.float32, "loss"),
                                   _ptr(dO, dO.dtype if dO is not None and dO.dtype == torch.bfloat16 else torch.float32, "dO"),
                                   _dt(dO, "dO"), dO.stride(0) if dO is not None else 0, _ptr(dO_colsum, torch.float32, "dO_colsum"),
                                   _stream(stream)))


def sgnn_spmm(ctx: Context, A: Csr, X: torch.Tensor, out: torch.Tensor, row_index: Optional[torch.Tensor] = None,
              stream=None, add: Optional[torch.Tensor] = None):
    """out = A X (+ add)."""
    a = A.struct()
    x, o = _mat(X, row_index, "X", allow_bf16=True), _mat(out, None, "out", allow_bf16=True)
    ad = _mat(add, None, "add") if add is not None else None
    ctx.check(lib().sgnn_spmm(ctx._h, C.byref(a), C.byref(x), C.byref(ad) if ad is not None else None, C.byref(o),
                              _stream(stream)))


def _flat(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise ValueError("%s must be a contiguous float32 tensor" % name)
    return t


def sgnn_sgd_step(ctx: Context, w: torch.Tensor, g: torch.Tensor, lr: float, weight_decay: float = 0.0, stream=None):
    """w <- w - lr (g + weight_decay w), in place."""
    _flat(w, "w"); _flat(g, "g")
    if g.numel() != w.numel():
        raise ValueError("g must have as many elements as w")
    ctx.check(lib().sgnn_sgd_step(ctx._h, w.data_ptr(), g.data_ptr(), w.numel(), lr, weight_decay, _stream(stream)))


def sgnn_adam_step(ctx: Context, w: torch.Tensor, g: torch.Tensor, m: torch.Tensor, v: torch.Tensor, lr: float, t: int,
                   beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, stream=None):
    """One Adam update of w in place; m, v are the moment buffers, t = 1, 2, ... the step number."""
    for x, nm in ((w, "w"), (g, "g"), (m, "m"), (v, "v")):
        _flat(x, nm)
        if x.numel() != w.numel():
            raise ValueError("%s must have as many elements as w" % nm)
    ctx.check(lib().sgnn_adam_step(ctx._h, w.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr(), w.numel(), lr, beta1,
                                   beta2, eps, t, _stream(stream)))


def _dt(t: Optional[torch.Tensor], name: str) -> int:
    if t is None or t.dtype == torch.float32:
        return SGNN_F32
    if t.dtype == torch.bfloat16:
        return SGNN_BF16
    raise TypeError("%s must be float32 or bfloat16, got %s" % (name, t.dtype))


def sgnn_gemm(ctx: Context, trans_a: bool, trans_b: bool, A: torch.Tensor, B: torch.Tensor, bias: Optional[torch.Tensor],
              flags: int, Cm: torch.Tensor, stream=None, b_colsum: Optional[torch.Tensor] = None,
              mask: Optional[torch.Tensor] = None):
    """C = act(op(A) op(B) + bias), zero where mask <= 0 (mask: a matrix shaped like C); b_colsum: column sums of B.
    A, B, C and the mask may be bfloat16 tensors (with SGNN_BF16_MFMA)."""
    M, N = Cm.shape
    if mask is not None and tuple(mask.shape) != (M, N):
        raise ValueError("mask must have the shape of C")
    K = A.shape[0] if trans_a else A.shape[1]
    ctx.check(lib().sgnn_gemm(ctx._h, int(trans_a), int(trans_b), M, N, K, _ptr(A, None, "A"), _dt(A, "A"), A.stride(0),
                              _ptr(B, None, "B"), _dt(B, "B"), B.stride(0), _ptr(bias, torch.float32, "bias"), flags,
                              _ptr(Cm, None, "C"), _dt(Cm, "C"), Cm.stride(0), _ptr(mask, None, "mask"), _dt(mask, "mask"),
                              mask.stride(0) if mask is not None else 0, _ptr(b_colsum, torch.float32, "b_colsum"),
                              _stream(stream)))


def sgnn_copy_f32(ctx: Context, src: torch.Tensor, dst: torch.Tensor, stream=None):
    ctx.check(lib().sgnn_copy_f32(ctx._h, _ptr(src, torch.float32, "src"), _ptr(dst, torch.float32, "dst"), src.numel(),
                                  _stream(stream)))
