"""Shards of the mini-batch matrix (Algorithm 2's row and column ranges) and the transposed build, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si
from gpu_util import DEV, TOL_VAL, ctx, gpu_sample
from helpers import rel_err

pytestmark = pytest.mark.gpu


def _sample(g, B, seed, step):
    S = oracle.sample_uniform(g.N, B, seed, step)
    W = (g.N + 63) // 64
    Sd = torch.empty(B, dtype=torch.int32, device=DEV); bm = torch.empty(W, dtype=torch.int64, device=DEV)
    rk = torch.empty(W, dtype=torch.int32, device=DEV)
    sg.sgnn_sample_uniform(ctx(), g.N, B, seed, step, Sd, bm, rk)
    assert np.array_equal(Sd.cpu().numpy(), S)
    return S, Sd, bm, rk


@pytest.mark.parametrize("B", [700, 4096])
def test_shards_match_oracle_and_tile_the_matrix(tiny_graph, B):
    g = tiny_graph
    rpg, cig = g.rowptr.numpy(), g.colidx.numpy()
    E = len(cig)
    ctx().reserve(g.N, E, B, 8, E)
    S, Sd, bm, rk = _sample(g, B, 5, 2)
    rpd, cid = g.rowptr.to(DEV), g.colidx.to(DEV)
    full = oracle.induced_csr(g.N, rpg, cig, S)
    cuts_r = [0, 1000, 1001, 2500, g.N]
    cuts_c = [0, 17, 3000, g.N]
    total = 0
    for a, b in zip(cuts_r[:-1], cuts_r[1:]):
        for c, d in zip(cuts_c[:-1], cuts_c[1:]):
            out = sg.Csr(B, B, E, DEV)
            nnz = sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, a, b, c, d, out, want_nnz=True)
            rpt, cit, vt = oracle.induced_csr_range(g.N, rpg, cig, S, a, b, c, d)
            assert nnz == len(cit)
            assert np.array_equal(out.rowptr.cpu().numpy(), rpt)
            assert np.array_equal(out.colidx.cpu().numpy()[:nnz], cit)
            if nnz:
                assert rel_err(out.val.cpu().numpy()[:nnz], vt) < TOL_VAL
            total += nnz
    assert total == len(full[1])
    # the whole ranges give the plain call, bit for bit
    o1 = sg.Csr(B, B, E, DEV); o2 = sg.Csr(B, B, E, DEV)
    n1 = sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, 0, g.N, 0, g.N, o1, want_nnz=True)
    n2 = sg.sgnn_induced_csr(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, o2, want_nnz=True)
    assert n1 == n2 and torch.equal(o1.rowptr, o2.rowptr) and torch.equal(o1.colidx[:n1], o2.colidx[:n1])
    assert torch.equal(o1.val[:n1], o2.val[:n1])
    # empty ranges and bad ranges
    o3 = sg.Csr(B, B, E, DEV)
    assert sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, 50, 50, 0, g.N, o3, want_nnz=True) == 0
    assert torch.all(o3.rowptr == 0)
    with pytest.raises(sg.SgnnError):
        sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, 0, g.N + 1, 0, g.N, o3)
    ctx().status()


def test_transpose_of_a_shard_and_of_a_directed_matrix(tiny_graph):
    g = tiny_graph
    rpg, cig = g.rowptr.numpy(), g.colidx.numpy()
    B = 2048; E = len(cig)
    ctx().reserve(g.N, E, B, 64, E)
    S, Sd, bm, rk = _sample(g, B, 9, 1)
    rpd, cid = g.rowptr.to(DEV), g.colidx.to(DEV)
    # a non-square shard: rows in [0, 1500), columns in [1200, N)
    A = sg.Csr(B, B, E, DEV)
    nnz = sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, 0, 1500, 1200, g.N, A, want_nnz=True)
    AT = sg.Csr(B, B, E, DEV)
    sg.sgnn_csr_transpose(ctx(), A, AT)
    rpt, cit, vt = oracle.induced_csr_range(g.N, rpg, cig, S, 0, 1500, 1200, g.N)
    rT, cT, vT = oracle.csr_transpose(B, B, rpt, cit, vt)
    assert AT.nnz() == nnz == len(cT)
    assert np.array_equal(AT.rowptr.cpu().numpy(), rT)
    assert np.array_equal(AT.colidx.cpu().numpy()[:nnz], cT)
    assert rel_err(AT.val.cpu().numpy()[:nnz], vT) < TOL_VAL
    # for an undirected graph that transpose is the shard with the ranges swapped
    A2 = sg.Csr(B, B, E, DEV)
    n2 = sg.sgnn_induced_csr_range(ctx(), g.N, rpd, cid, None, Sd, B, bm, rk, 1200, g.N, 0, 1500, A2, want_nnz=True)
    assert n2 == nnz and torch.equal(A2.rowptr, AT.rowptr) and torch.equal(A2.colidx[:nnz], AT.colidx[:nnz])
    assert torch.equal(A2.val[:nnz], AT.val[:nnz])
    # the backward product through the transposed shard
    X = np.random.default_rng(1).standard_normal((B, 64)).astype(np.float32)
    out = torch.zeros((B, 64), dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), AT, torch.tensor(X, device=DEV), out)
    assert rel_err(out.cpu().numpy(), oracle.spmm(rT, cT, vT, X)) < 1e-5
    # a rectangular, directed matrix with one long row and one long column, twice (same bits)
    rng = np.random.default_rng(3)
    rows, cols = 300, 500
    dense = (rng.random((rows, cols)) < 0.02) * rng.standard_normal((rows, cols))
    dense[7, :] = rng.standard_normal(cols); dense[:, 11] = rng.standard_normal(rows)
    rp = [0]; ci = []; v = []
    for i in range(rows):
        nz = np.nonzero(dense[i])[0]
        ci += list(nz); v += list(dense[i, nz].astype(np.float32)); rp.append(len(ci))
    M = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV)
    MT = sg.Csr(cols, rows, len(ci), DEV); MT2 = sg.Csr(cols, rows, len(ci), DEV)
    sg.sgnn_csr_transpose(ctx(), M, MT); sg.sgnn_csr_transpose(ctx(), M, MT2)
    rT, cT, vT = oracle.csr_transpose(rows, cols, np.array(rp, np.int32), np.array(ci, np.int32), np.array(v, np.float32))
    assert np.array_equal(MT.rowptr.cpu().numpy(), rT) and np.array_equal(MT.colidx.cpu().numpy()[:len(cT)], cT)
    assert np.array_equal(MT.val.cpu().numpy()[:len(cT)], vT)
    assert torch.equal(MT.colidx, MT2.colidx) and torch.equal(MT.val, MT2.val)
    ctx().status()


def test_transpose_rows_of_every_length_class():
    """Columns with a handful of entries (ranked by one thread), with a few hundred (by a wavefront) and
    hub columns ranked through the bitmap over the source rows, here wider than one bitmap window."""
    rng = np.random.default_rng(21)
    rows, cols = 150000, 1500
    per_row = rng.integers(0, 3, rows)
    r_idx = np.repeat(np.arange(rows), per_row)
    c_idx = rng.integers(20, cols, len(r_idx))
    extra = []
    for col, n in ((3, 17), (4, 300), (5, 512), (6, 513), (7, 6000), (8, 40000), (300, 2500)):
        extra.append((np.sort(rng.choice(rows, n, replace=False)), np.full(n, col)))
    r_idx = np.concatenate([r_idx] + [e[0] for e in extra]); c_idx = np.concatenate([c_idx] + [e[1] for e in extra])
    key = np.unique(r_idx.astype(np.int64) * cols + c_idx)          # a row holds a column once, in ascending order
    r_idx, c_idx = (key // cols).astype(np.int64), (key % cols).astype(np.int32)
    rp = np.zeros(rows + 1, np.int32); np.add.at(rp, r_idx + 1, 1); rp = np.cumsum(rp).astype(np.int32)
    v = rng.standard_normal(len(c_idx)).astype(np.float32)
    ctx().reserve(rows, len(c_idx), max(rows, cols), 8, len(c_idx))
    M = sg.Csr.from_arrays(rows, cols, rp, c_idx, v, DEV)
    MT = sg.Csr(cols, rows, len(c_idx), DEV)
    sg.sgnn_csr_transpose(ctx(), M, MT)
    rT, cT, vT = oracle.csr_transpose(rows, cols, rp, c_idx, v)
    assert np.array_equal(MT.rowptr.cpu().numpy(), rT)
    assert np.array_equal(MT.colidx.cpu().numpy()[:len(cT)], cT)
    assert np.array_equal(MT.val.cpu().numpy()[:len(cT)], vT)
    ctx().status()
