"""Independent small reference routines used to pin the oracle (numpy / pure Python)."""
import itertools
import math

import numpy as np

M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox_py(ctr, key, rounds=10):
    """Philox4x32 on Python integers, written from the round description in the SC'11 paper:
    two 32x32->64 products; new = (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))."""
    c = [int(x) & MASK for x in ctr]
    k = [int(x) & MASK for x in key]
    for _ in range(rounds):
        a = M0 * c[0]
        b = M1 * c[2]
        c = [((b >> 32) ^ c[1] ^ k[0]) & MASK, b & MASK, ((a >> 32) ^ c[3] ^ k[1]) & MASK, a & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def vertex_key_py(seed, step, v):
    j = v >> 1
    out = philox_py([j & MASK, j >> 32, step & MASK, step >> 32], [seed & MASK, seed >> 32])
    return (out[1] << 32 | out[0]) if v % 2 == 0 else (out[3] << 32 | out[2])


def dense_normalized(N, rowptr, colidx):
    """Dense D^-1/2 (A+I) D^-1/2 (Eq. 3) from the canonical CSR of A+I."""
    A = np.zeros((N, N))
    for v in range(N):
        A[v, colidx[rowptr[v]:rowptr[v + 1]]] = 1.0
    deg = A.sum(1)
    return A / np.sqrt(np.outer(deg, deg)), A


def dense_induced(N, rowptr, colidx, S, norm_mode=0, rescale=1):
    """Dense brute force of Eqs. 21-24: take [S,S], rescale the off-diagonal by 1/p."""
    An, A01 = dense_normalized(N, rowptr, colidx)
    S = np.asarray(S)
    B = len(S)
    if norm_mode == 0:
        sub = An[np.ix_(S, S)].copy()
    else:
        m = A01[np.ix_(S, S)]
        deg = m.sum(1)
        sub = m / np.sqrt(np.outer(deg, deg))
    if rescale and B > 1:
        p = (B - 1) / (N - 1)
        off = ~np.eye(B, dtype=bool)
        sub[off] /= p
    return sub


def csr_to_dense(rowptr, colidx, val, ncols):
    rows = len(rowptr) - 1
    D = np.zeros((rows, ncols))
    for i in range(rows):
        for e in range(rowptr[i], rowptr[i + 1]):
            D[i, colidx[e]] += val[e]
    return D


def algorithm2_literal(N, rowptr, colidx, val, S, rescale=1):
    """Walk through the four phases of Algorithm 2 (full row and column range) with numpy
    array primitives: row lengths, prefix sum, owner search, gather, membership, remap, rescale."""
    S = np.asarray(S, np.int64)
    B = len(S)
    r = rowptr[S + 1] - rowptr[S]
    P = np.cumsum(r)
    total = int(P[-1])
    flat = np.arange(total)
    own = np.searchsorted(P, flat, side="right")
    start = P - r
    e = rowptr[S[own]] + (flat - start[own])
    i_g = S[own]
    j_g = colidx[e].astype(np.int64)
    v_e = val[e].astype(np.float64)
    mask = np.isin(j_g, S)
    i_g, j_g, v_e = i_g[mask], j_g[mask], v_e[mask]
    remap = np.full(N, -1, np.int64)
    remap[S] = np.arange(B)
    i_c, j_c = remap[i_g], remap[j_g]
    if rescale and B > 1:
        p = (B - 1) / (N - 1)
        v_e = np.where(i_g != j_g, v_e / p, v_e)
    order = np.lexsort((j_c, i_c))
    i_c, j_c, v_e = i_c[order], j_c[order], v_e[order]
    rp = np.zeros(B + 1, np.int64)
    np.add.at(rp, i_c + 1, 1)
    return np.cumsum(rp), j_c, v_e


def rel_err(got, ref):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    nref = np.linalg.norm(ref)
    fro = np.linalg.norm(got - ref) / (nref if nref > 0 else 1.0)
    mref = np.abs(ref).max() if ref.size else 0.0
    mx = (np.abs(got - ref).max() if ref.size else 0.0) / (mref if mref > 0 else 1.0)
    return max(fro, mx)
