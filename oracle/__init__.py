"""CPU oracle of the mini-batch GCN hot path: ctypes front end to sgnn_oracle.c.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; the product package never imports it and it never imports the product.
All arrays are numpy arrays on the host.  See the header of sgnn_oracle.c for the passages of
the paper each routine follows and for how each is pinned.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sgnn_oracle.c")
_LIB = os.path.join(_HERE, "libsgnn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sgnn_oracle.c with gcc (OpenMP over independent outer loops only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u32p, i32p, i64p, f32p, f64p, u64p = (C.POINTER(t) for t in
                                              (C.c_uint32, C.c_int32, C.c_int64, C.c_float, C.c_double, C.c_uint64))
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_vertex_key.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.oracle_vertex_key.restype = C.c_uint64
        L.oracle_vertex_keys.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, u64p]
        L.oracle_vertex_keys.restype = None
        L.oracle_sample_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64, i32p]
        L.oracle_sample_uniform.restype = C.c_int
        L.oracle_induced_csr.argtypes = [C.c_uint64, i64p, i32p, f32p, i32p, C.c_uint64, C.c_int, C.c_int,
                                         i32p, i32p, f32p, C.c_int64]
        L.oracle_induced_csr.restype = C.c_int64
        L.oracle_gather_rows.argtypes = [f32p, C.c_int64, i32p, C.c_int64, f64p]
        L.oracle_gather_rows.restype = None
        L.oracle_gather_labels.argtypes = [i32p, i32p, C.c_int64, i32p]
        L.oracle_gather_labels.restype = None
        L.oracle_round_bf16.argtypes = [C.c_double]
        L.oracle_round_bf16.restype = C.c_double
        L.oracle_spmm.argtypes = [C.c_int64, i32p, i32p, f32p, f64p, C.c_int64, f64p]
        L.oracle_spmm.restype = None
        L.oracle_csr_transpose.argtypes = [C.c_int64, C.c_int64, i32p, i32p, f32p, i32p, i32p, f32p]
        L.oracle_csr_transpose.restype = None
        L.oracle_gemm.argtypes = [C.c_int64, C.c_int64, C.c_int64, f64p, f64p, f64p]
        L.oracle_gemm.restype = None
        L.oracle_gcn_fwd.argtypes = [C.c_int64, i32p, i32p, f32p, f64p, C.c_int64, f64p, C.c_int64, f64p,
                                     C.c_int, C.c_int, f64p, f64p]
        L.oracle_gcn_fwd.restype = None
        L.oracle_gcn_bwd.argtypes = [C.c_int64, i32p, i32p, f32p, f64p, C.c_int64, f64p, C.c_int64, f64p, f64p,
                                     C.c_int, C.c_int, f64p, f64p, f64p]
        L.oracle_gcn_bwd.restype = None
        L.oracle_softmax_xent.argtypes = [C.c_int64, C.c_int64, f64p, i32p, f64p]
        L.oracle_softmax_xent.restype = C.c_double
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _arr(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


# ------------------------------------------------------------------------------------------------

def philox4x32_10(ctr, key) -> np.ndarray:
    c = _arr(ctr, np.uint32); k = _arr(key, np.uint32); out = np.zeros(4, np.uint32)
    lib().oracle_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def vertex_key(seed: int, step: int, v: int) -> int:
    return int(lib().oracle_vertex_key(seed, step, v))


def vertex_keys(seed: int, step: int, N: int) -> np.ndarray:
    out = np.zeros(N, np.uint64)
    lib().oracle_vertex_keys(seed, step, N, _p(out, C.c_uint64))
    return out


def sample_uniform(N: int, B: int, seed: int, step: int) -> np.ndarray:
    """Eq. 20: ascending int32[B]."""
    S = np.zeros(max(B, 1), np.int32)
    rc = lib().oracle_sample_uniform(N, B, seed, step, _p(S, C.c_int32))
    if rc != 0:
        raise ValueError("oracle_sample_uniform: invalid arguments")
    return S[:B]


def induced_csr(N: int, rowptr, colidx, S, val=None, norm_mode: int = 0, rescale: int = 1
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eqs. 21-24: (rowptr_S int32[B+1], colidx_S int32[nnz], val_S float32[nnz])."""
    rp = _arr(rowptr, np.int64); ci = _arr(colidx, np.int32); S = _arr(S, np.int32)
    vv = None if val is None else _arr(val, np.float32)
    B = int(S.shape[0])
    cap = int(sum(int(rp[v + 1] - rp[v]) for v in S.tolist())) if B < 200000 else int((rp[S.astype(np.int64) + 1] - rp[S.astype(np.int64)]).sum())
    cap = max(cap, 1)
    rpS = np.zeros(B + 1, np.int32); ciS = np.zeros(cap, np.int32); vS = np.zeros(cap, np.float32)
    nnz = lib().oracle_induced_csr(N, _p(rp, C.c_int64), _p(ci, C.c_int32), _p(vv, C.c_float), _p(S, C.c_int32), B,
                                   norm_mode, rescale, _p(rpS, C.c_int32), _p(ciS, C.c_int32), _p(vS, C.c_float), cap)
    if nnz < 0:
        raise ValueError("oracle_induced_csr: invalid arguments")
    return rpS, ciS[:nnz].copy(), vS[:nnz].copy()


def induced_csr_range(N: int, rowptr, colidx, S, R0: int, R1: int, C0: int, C1: int, val=None, rescale: int = 1):
    """Algorithm 2 for one shard: rows of S in [R0, R1), columns of S in [C0, C1); B x B namespace."""
    rp = _arr(rowptr, np.int64); ci = _arr(colidx, np.int32); S = _arr(S, np.int32)
    vv = None if val is None else _arr(val, np.float32)
    B = int(S.shape[0])
    cap = max(int((rp[S.astype(np.int64) + 1] - rp[S.astype(np.int64)]).sum()), 1)
    rpS = np.zeros(B + 1, np.int32); ciS = np.zeros(cap, np.int32); vS = np.zeros(cap, np.float32)
    L = lib()
    L.oracle_induced_csr_range.restype = C.c_int64
    L.oracle_induced_csr_range.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_int,
                                           C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int64]
    nnz = L.oracle_induced_csr_range(N, rp.ctypes.data, ci.ctypes.data, vv.ctypes.data if vv is not None else None,
                                     S.ctypes.data, B, rescale, R0, R1, C0, C1, rpS.ctypes.data, ciS.ctypes.data,
                                     vS.ctypes.data, cap)
    if nnz < 0:
        raise ValueError("oracle_induced_csr_range: invalid arguments")
    return rpS, ciS[:nnz].copy(), vS[:nnz].copy()


def gather_rows(X, S) -> np.ndarray:
    X = _arr(X, np.float32); S = _arr(S, np.int32)
    out = np.zeros((S.shape[0], X.shape[1]), np.float64)
    lib().oracle_gather_rows(_p(X, C.c_float), X.shape[1], _p(S, C.c_int32), S.shape[0], _p(out, C.c_double))
    return out


def gather_labels(Y, S) -> np.ndarray:
    Y = _arr(Y, np.int32); S = _arr(S, np.int32)
    out = np.zeros(S.shape[0], np.int32)
    lib().oracle_gather_labels(_p(Y, C.c_int32), _p(S, C.c_int32), S.shape[0], _p(out, C.c_int32))
    return out


def round_bf16(x):
    """Every element rounded to bfloat16 (nearest, ties to even), returned as float64."""
    a = np.ascontiguousarray(x, np.float64)
    out = np.empty_like(a)
    L = lib()
    L.oracle_round_bf16_array.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
    L.oracle_round_bf16_array.restype = None
    L.oracle_round_bf16_array(a.ctypes.data, out.ctypes.data, a.size)
    return out


def spmm(rowptr, colidx, val, H) -> np.ndarray:
    rp = _arr(rowptr, np.int32); ci = _arr(colidx, np.int32); v = _arr(val, np.float32); H = _arr(H, np.float64)
    rows = rp.shape[0] - 1
    out = np.zeros((rows, H.shape[1]), np.float64)
    lib().oracle_spmm(rows, _p(rp, C.c_int32), _p(ci, C.c_int32), _p(v, C.c_float), _p(H, C.c_double), H.shape[1],
                      _p(out, C.c_double))
    return out


def csr_transpose(rows: int, cols: int, rowptr, colidx, val):
    rp = _arr(rowptr, np.int32); ci = _arr(colidx, np.int32); v = _arr(val, np.float32)
    rpT = np.zeros(cols + 1, np.int32); ciT = np.zeros(max(ci.shape[0], 1), np.int32)
    vT = np.zeros(max(ci.shape[0], 1), np.float32)
    lib().oracle_csr_transpose(rows, cols, _p(rp, C.c_int32), _p(ci, C.c_int32), _p(v, C.c_float),
                               _p(rpT, C.c_int32), _p(ciT, C.c_int32), _p(vT, C.c_float))
    return rpT, ciT[:ci.shape[0]], vT[:ci.shape[0]]


def gemm(A, Bm) -> np.ndarray:
    A = _arr(A, np.float64); Bm = _arr(Bm, np.float64)
    out = np.zeros((A.shape[0], Bm.shape[1]), np.float64)
    lib().oracle_gemm(A.shape[0], A.shape[1], Bm.shape[1], _p(A, C.c_double), _p(Bm, C.c_double), _p(out, C.c_double))
    return out


def gcn_fwd(rowptr, colidx, val, H, W, bias=None, relu: bool = True, bf16: bool = False):
    """Returns (T = A_S H, Y = act(T W + b)), both float64."""
    rp = _arr(rowptr, np.int32); ci = _arr(colidx, np.int32); v = _arr(val, np.float32)
    H = _arr(H, np.float64); W = _arr(W, np.float64)
    b = None if bias is None else _arr(bias, np.float64)
    B = rp.shape[0] - 1
    T = np.zeros((B, W.shape[0]), np.float64); Y = np.zeros((B, W.shape[1]), np.float64)
    lib().oracle_gcn_fwd(B, _p(rp, C.c_int32), _p(ci, C.c_int32), _p(v, C.c_float), _p(H, C.c_double), W.shape[0],
                         _p(W, C.c_double), W.shape[1], _p(b, C.c_double), int(relu), int(bf16),
                         _p(T, C.c_double), _p(Y, C.c_double))
    return T, Y


def gcn_bwd(rowptr_T, colidx_T, val_T, T, W, Y, dY, relu: bool = True, bf16: bool = False, need_dH: bool = True,
            store_dT_bf16: bool = False):
    """Returns (dH or None, dW, db), float64.  store_dT_bf16: dT = dZ W^T is rounded to bfloat16 (as
    stored) before dH = A^T dT."""
    rp = _arr(rowptr_T, np.int32); ci = _arr(colidx_T, np.int32); v = _arr(val_T, np.float32)
    T = _arr(T, np.float64); W = _arr(W, np.float64); Y = _arr(Y, np.float64); dY = _arr(dY, np.float64)
    B = rp.shape[0] - 1
    dH = np.zeros((B, W.shape[0]), np.float64) if need_dH else None
    dW = np.zeros_like(W); db = np.zeros(W.shape[1], np.float64)
    lib().oracle_gcn_bwd(B, _p(rp, C.c_int32), _p(ci, C.c_int32), _p(v, C.c_float), _p(T, C.c_double), W.shape[0],
                         _p(W, C.c_double), W.shape[1], _p(Y, C.c_double), _p(dY, C.c_double), int(relu), int(bool(bf16)) | (2 if store_dT_bf16 else 0),
                         _p(dH, C.c_double), _p(dW, C.c_double), _p(db, C.c_double))
    return dH, dW, db


def softmax_xent(O, labels):
    """Returns (mean loss, dO)."""
    O = _arr(O, np.float64); y = _arr(labels, np.int32)
    dO = np.zeros_like(O)
    loss = lib().oracle_softmax_xent(O.shape[0], O.shape[1], _p(O, C.c_double), _p(y, C.c_int32), _p(dO, C.c_double))
    return float(loss), dO


def dropout_keep(seed: int, layer: int, step: int, n_elems: int, q: float) -> np.ndarray:
    """Boolean keep mask of the first n_elems elements of a layer (row-major element numbering)."""
    L = lib()
    L.oracle_dropout_mask.restype = None
    L.oracle_dropout_mask.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64, C.c_double, C.c_void_p]
    out = np.zeros(n_elems, np.uint8)
    L.oracle_dropout_mask(seed, layer, step, n_elems, q, out.ctypes.data)
    return out.astype(bool)


def tail_fwd(Z, gamma=None, eps: float = 1e-6, R=None, q: float = 0.0, seed: int = 0, layer: int = 0, step: int = 0):
    """Y = dropout(relu(rmsnorm(Z; gamma, eps)), q) + R  (Eqs. 7-10).  Returns (Y, inv_rms, Xn), float64."""
    Z = _arr(Z, np.float64)
    g = None if gamma is None else _arr(gamma, np.float64)
    r = None if R is None else _arr(R, np.float64)
    Bn, d = Z.shape
    Y = np.zeros_like(Z); ir = np.zeros(Bn, np.float64); Xn = np.zeros_like(Z)
    L = lib()
    L.oracle_tail_fwd.restype = None
    L.oracle_tail_fwd.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p, C.c_double,
                                  C.c_uint64, C.c_uint32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
    L.oracle_tail_fwd(Bn, d, Z.ctypes.data, g.ctypes.data if g is not None else None, eps,
                      r.ctypes.data if r is not None else None, q, seed, layer, step, Y.ctypes.data, ir.ctypes.data,
                      Xn.ctypes.data)
    return Y, ir, Xn


def tail_bwd(Z, dY, gamma=None, eps: float = 1e-6, q: float = 0.0, seed: int = 0, layer: int = 0, step: int = 0):
    """Backward of the main branch of the layer tail.  Returns (dZ, dgamma), float64."""
    Z = _arr(Z, np.float64); dY = _arr(dY, np.float64)
    g = None if gamma is None else _arr(gamma, np.float64)
    Bn, d = Z.shape
    dZ = np.zeros_like(Z); dg = np.zeros(d, np.float64)
    L = lib()
    L.oracle_tail_bwd.restype = None
    L.oracle_tail_bwd.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_double, C.c_double, C.c_uint64,
                                  C.c_uint32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
    L.oracle_tail_bwd(Bn, d, Z.ctypes.data, g.ctypes.data if g is not None else None, eps, q, seed, layer, step,
                      dY.ctypes.data, dZ.ctypes.data, dg.ctypes.data)
    return dZ, dg


def sgd_step(w, g, lr: float, weight_decay: float = 0.0) -> np.ndarray:
    """w - lr (g + weight_decay w): the plain gradient step (Alg. 1 line 7 names no optimizer)."""
    w = _arr(w, np.float64); g = _arr(g, np.float64)
    return w - lr * (g + weight_decay * w)


def adam_step(w, g, m, v, lr: float, t: int, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8):
    """One step of Adam (Kingma & Ba, ICLR 2015, Algorithm 1), t = 1, 2, ...  Returns (w, m, v)."""
    w = _arr(w, np.float64); g = _arr(g, np.float64); m = _arr(m, np.float64); v = _arr(v, np.float64)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v


def model_step(rowptr, colidx, val, X_S, y_S, params, drop_q: float = 0.0, drop_seed: int = 0, step: int = 0,
               eps: float = 1e-6, bf16: bool = False):
    """The paper's complete model on one mini-batch (Fig. 2; Sec. III-B, III-C), forward and backward:
        X_h0 = X_S W_in;  for l = 1..L:  T_l = A X_h,l-1,  Z_l = T_l W_l,
        X_h,l = dropout(relu(rmsnorm(Z_l; gamma_l))) + X_h,l-1;   O = X_h,L W_out;  mean cross-entropy.
    params = {"W_in": d_in x d_h, "layers": [(W_l d_h x d_h, gamma_l d_h), ...], "W_out": d_h x c}.
    Returns a dict with the loss, every activation and the gradient of every parameter (float64).
    bf16: GEMM operands rounded to bfloat16 as in gcn_fwd / gcn_bwd."""
    rp = _arr(rowptr, np.int32); ci = _arr(colidx, np.int32); v = _arr(val, np.float32)
    Bn = rp.shape[0] - 1
    rd = (lambda a: round_bf16(a)) if bf16 else (lambda a: _arr(a, np.float64))
    X_S = _arr(X_S, np.float64)
    W_in = _arr(params["W_in"], np.float64); W_out = _arr(params["W_out"], np.float64)
    Xh = [gemm(rd(X_S), rd(W_in))]
    T, Z, IR = [], [], []
    for l, (W, gam) in enumerate(params["layers"]):
        T.append(spmm(rp, ci, v, Xh[-1]))                                    # Eq. 5
        Z.append(gemm(rd(T[-1]), rd(W)))                                     # Eq. 6
        Y, ir, _ = tail_fwd(Z[-1], gamma=gam, eps=eps, R=Xh[-1], q=drop_q, seed=drop_seed, layer=l, step=step)   # Eqs. 7-10
        Xh.append(Y); IR.append(ir)
    O = gemm(rd(Xh[-1]), rd(W_out))
    loss, dO = softmax_xent(O, y_S)
    out = {"Xh": Xh, "T": T, "Z": Z, "inv_rms": IR, "O": O, "loss": loss, "dO": dO}
    # backward (Sec. III-C)
    out["dW_out"] = gemm(rd(Xh[-1]).T.copy(), rd(dO))
    dX = gemm(rd(dO), rd(W_out).T.copy())
    rpT, ciT, vT = csr_transpose(Bn, Bn, rp, ci, v)
    dWs, dgs = [None] * len(Z), [None] * len(Z)
    for l in range(len(Z) - 1, -1, -1):
        W, gam = params["layers"][l]
        dZ, dg = tail_bwd(Z[l], dX, gamma=gam, eps=eps, q=drop_q, seed=drop_seed, layer=l, step=step)
        dWs[l] = gemm(rd(T[l]).T.copy(), rd(dZ)); dgs[l] = dg
        dT = gemm(rd(dZ), rd(_arr(W, np.float64)).T.copy())
        dX = spmm(rpT, ciT, vT, dT) + dX                                     # conv path + skip path
    out["dW"] = dWs; out["dgamma"] = dgs
    out["dW_in"] = gemm(rd(X_S).T.copy(), rd(dX)); out["dXh0"] = dX
    return out


def sigmoid_bce(O, Y):
    """Mean binary cross-entropy on logits and its gradient.  Returns (loss, dO)."""
    O = _arr(O, np.float64); Y = _arr(Y, np.float64)
    dO = np.zeros_like(O)
    L = lib()
    L.oracle_sigmoid_bce.restype = C.c_double
    L.oracle_sigmoid_bce.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    return float(L.oracle_sigmoid_bce(O.shape[0], O.shape[1], O.ctypes.data, Y.ctypes.data, dO.ctypes.data)), dO


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def gcn_step(N, rowptr, colidx, X, labels, weights, B, seed, step, bf16=False, norm_mode=0, rescale=1,
             relu_ties=None, tie_band=0.0, store_bf16=False, dO_ties=None, logit_band=0.0, grad_band=None):
    """One whole mini-batch step (Algorithm 1 without the parameter update): sample, induce,
    slice, L layers forward (ReLU on all but the last), mean cross-entropy, L layers backward.
    `weights` is a list of (W, b).  Returns a dict of every intermediate, float64.

    ReLU ties: a pre-activation within tie_band * max|Z| of zero has no decidable sign at the
    working precision, and either mask value is a correct result there.  relu_ties[l], when
    given, is a boolean B x d_out array; inside that band (and only there) the backward mask of
    layer l takes its value instead of the oracle's own Z > 0.  The forward values never change.
    store_bf16, dO_ties, logit_band: see layers_step."""
    S = sample_uniform(N, B, seed, step)
    rpS, ciS, vS = induced_csr(N, rowptr, colidx, S, None, norm_mode, rescale)
    H = gather_rows(X, S)
    yS = gather_labels(labels, S)
    out = layers_step(rpS, ciS, vS, H, yS, weights, bf16=bf16, relu_ties=relu_ties, tie_band=tie_band,
                      store_bf16=store_bf16, dO_ties=dO_ties, logit_band=logit_band, grad_band=grad_band)
    out["S"] = S
    return out


def undecidable_loss_rows(O, labels, logit_band, grad_band=None):
    """Rows of the logits O whose cross-entropy gradient row is not decidable at a relative logit
    accuracy of logit_band, to within grad_band (default: the same figure).

    With every logit of row i known to within eps_i = logit_band * max_j |O_ij|, a probability
    p_j = softmax(O_i)_j lies between p_j e^(-2 eps_i) and p_j e^(2 eps_i), and so does 1 - p_j with
    respect to itself; entry j of the gradient row (softmax(O_i) - onehot(y_i)) / B can therefore move
    by at most min(p_j, 1 - p_j) (e^(2 eps_i) - 1) / B.  The row is undecidable when that bound, taken
    over its entries, exceeds grad_band times the largest gradient entry of the whole batch (the
    scale the weight gradients are measured on): large logits whose leading probabilities are not
    saturated.  Rows with small logits, and rows with one dominant class, are decidable."""
    O = np.asarray(O, np.float64)
    if logit_band <= 0.0:
        return np.zeros(O.shape[0], bool)
    if grad_band is None:
        grad_band = logit_band
    m = O.max(axis=1, keepdims=True)
    e = np.exp(O - m)
    p = e / e.sum(axis=1, keepdims=True)
    eps = logit_band * np.abs(O).max(axis=1)
    onehot = np.zeros_like(p)
    onehot[np.arange(O.shape[0]), np.asarray(labels, np.int64)] = 1.0
    g = np.abs(p - onehot).max()
    q = np.minimum(p, 1.0 - p).max(axis=1)
    with np.errstate(over="ignore"):
        grow = np.expm1(2.0 * eps)
    bound = np.where(q > 0.0, q * np.where(np.isfinite(grow), grow, np.finfo(np.float64).max / 2), 0.0)
    return bound > grad_band * g


def layers_step(rpS, ciS, vS, X_S, y_S, weights, bf16=False, relu_ties=None, tie_band=0.0, store_bf16=False,
                dO_ties=None, logit_band=0.0, grad_band=None):
    """The layer part of a step on an already extracted mini-batch: L layers forward, mean
    cross-entropy, L layers backward (see gcn_step for relu_ties / tie_band).

    store_bf16: the activations H_l (l < L) are stored as bfloat16 between the layers (the reading
    taken for the configuration whose features and activations are bfloat16): they are rounded to
    nearest even once, after the activation, and everything downstream - the next aggregation, the
    ReLU mask - sees the stored value.  The aggregates T_l are GEMM operands and are rounded by
    bf16=True already; the logits H_L stay unrounded.  The gradient dH_l handed from layer l to layer
    l-1 is stored as bfloat16 too: the dense products of layer l-1 round it anyway, so the one thing
    that changes is that layer's bias gradient, which becomes the column sum of the rounded values.
    Inside a layer the gradient of the aggregate, dT_l = dZ_l W_l^T, is stored as bfloat16 as well (the
    mirror image of the forward pass, whose sparse product reads bfloat16 activations): it is rounded once
    before dH_l = A^T dT_l.  The loss gradient dO is stored as bfloat16 too: the last layer's bias gradient is
    the column sum of the rounded values, and its other products start from them (the returned "dO" is the
    unrounded one).  dZ stays unrounded.

    dO_ties, logit_band: the loss gradient has the same kind of undecidable set as the ReLU mask.
    Rows of the logits for which undecidable_loss_rows(H_L, y, logit_band) holds form the returned
    "dO_band"; inside it (and only there) the backward pass starts from the rows of dO_ties when
    given; every other row starts from the oracle's own gradient.  The forward values, the loss and
    the returned "dO" are always the oracle's own."""
    B = len(rpS) - 1
    H = np.ascontiguousarray(X_S, np.float64)
    yS = np.ascontiguousarray(y_S, np.int32)
    rpT, ciT, vT = csr_transpose(B, B, rpS, ciS, vS)
    L = len(weights)
    Ts, Hs, masks, bands = [], [H], [], []
    for l, (W, b) in enumerate(weights):
        relu = l < L - 1
        T, Z = gcn_fwd(rpS, ciS, vS, Hs[-1], W, b, relu=False, bf16=bf16)
        Y = np.maximum(Z, 0.0) if relu else Z
        mask = Z > 0.0
        band = np.abs(Z) <= tie_band * np.abs(Z).max() if relu else np.zeros_like(mask)
        if relu and relu_ties is not None and relu_ties[l] is not None:
            mask = np.where(band, np.asarray(relu_ties[l], bool), mask)
        if relu and store_bf16:
            Y = round_bf16(Y)
        Ts.append(T); Hs.append(Y); masks.append(mask); bands.append(band)
    loss, dY = softmax_xent(Hs[-1], yS)
    dO_own = dY
    dO_band = undecidable_loss_rows(Hs[-1], yS, logit_band, grad_band)
    if dO_ties is not None and dO_band.any():
        dY = dY.copy()
        dY[dO_band] = np.asarray(dO_ties, np.float64)[dO_band]
    dWs, dbs, dHs = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        W, b = weights[l]
        relu = l < L - 1
        if store_bf16:
            # dO (l = L-1) and dH_{l+1} as stored (the ReLU mask is 0 / 1: rounding before or after it is the same)
            dY = round_bf16(dY)
        Ymask = masks[l].astype(np.float64) if relu else Hs[l + 1]     # gcn_bwd only tests Y > 0
        dH, dW, db = gcn_bwd(rpT, ciT, vT, Ts[l], W, Ymask, dY, relu=relu, bf16=bf16, need_dH=(l > 0),
                             store_dT_bf16=store_bf16)
        dWs[l], dbs[l], dHs[l] = dW, db, dH
        dY = dH
    return dict(rowptr=rpS, colidx=ciS, val=vS, X_S=H, y_S=yS, T=Ts, H=Hs, loss=loss, dO=dO_own, dO_band=dO_band, dW=dWs,
                db=dbs, dH=dHs, relu_band=bands, relu_mask=masks)
