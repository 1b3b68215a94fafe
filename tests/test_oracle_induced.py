"""Pins for the oracle's induced, normalised, rescaled subgraph (Eqs. 21-25, Algorithm 2)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth_inputs as si
from helpers import algorithm2_literal, csr_to_dense, dense_induced, dense_normalized


def _np_graph(g):
    return g.rowptr.numpy().astype(np.int64), g.colidx.numpy().astype(np.int32)


@pytest.fixture(scope="module")
def small():
    g = si.rmat_graph(300, 1500, seed=77)
    return (300,) + _np_graph(g)


def test_generator_gives_canonical_csr(small):
    N, rp, ci = small
    for v in range(N):
        row = ci[rp[v]:rp[v + 1]]
        assert np.all(np.diff(row) > 0) and v in row
    A = csr_to_dense(rp, ci, np.ones(len(ci)), N)
    assert np.array_equal(A, A.T)


@pytest.mark.parametrize("norm_mode", [0, 1])
@pytest.mark.parametrize("rescale", [0, 1])
@pytest.mark.parametrize("B", [1, 2, 37, 150, 300])
def test_against_dense_brute_force(small, B, rescale, norm_mode):
    N, rp, ci = small
    S = oracle.sample_uniform(N, B, 3, B)
    rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, None, norm_mode, rescale)
    ref = dense_induced(N, rp, ci, S, norm_mode, rescale)
    got = csr_to_dense(rpS, ciS, vS, B)
    # structure exactly, values to fp32 rounding
    assert np.array_equal(got != 0, ref != 0)
    assert np.allclose(got, ref, rtol=1e-6, atol=0)
    for i in range(B):
        assert np.all(np.diff(ciS[rpS[i]:rpS[i + 1]]) > 0)
    # edge count = number of (u,v) in E with both endpoints in S (Eq. 21)
    inS = np.zeros(N, bool); inS[S] = True
    cnt = sum(int(inS[ci[rp[v]:rp[v + 1]]].sum()) for v in S)
    assert len(ciS) == cnt == rpS[-1]


def test_against_scipy_slicing(small):
    N, rp, ci = small
    deg = np.diff(rp).astype(np.float64)
    val = (1.0 / np.sqrt(deg[np.repeat(np.arange(N), np.diff(rp))] * deg[ci])).astype(np.float32)
    A = sp.csr_matrix((val, ci, rp), shape=(N, N))
    S = oracle.sample_uniform(N, 120, 0, 0)
    sub = A[S][:, S].tocsr(); sub.sort_indices()
    rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, val, 0, 0)   # weights verbatim, no rescale
    assert np.array_equal(rpS, sub.indptr) and np.array_equal(ciS, sub.indices)
    assert np.array_equal(vS, sub.data)
    # and computing the weights from degrees gives the same numbers as passing them in
    rp2, ci2, v2 = oracle.induced_csr(N, rp, ci, S, None, 0, 0)
    assert np.array_equal(ci2, ciS) and np.allclose(v2, vS, rtol=1e-7)


def test_identity_extraction_when_all_vertices_sampled(small):
    N, rp, ci = small
    S = np.arange(N, dtype=np.int32)
    rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, None, 0, 1)   # p = 1
    assert np.array_equal(rpS, rp) and np.array_equal(ciS, ci)
    An, _ = dense_normalized(N, rp, ci)
    assert np.allclose(csr_to_dense(rpS, ciS, vS, N), An, rtol=1e-6)


def test_row_sums_and_symmetry(small):
    N, rp, ci = small
    S = oracle.sample_uniform(N, 100, 1, 1)
    for mode in (0, 1):
        rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, None, mode, 1)
        D = csr_to_dense(rpS, ciS, vS, 100)
        ref = dense_induced(N, rp, ci, S, mode, 1)
        assert np.allclose(D @ np.ones(100), ref @ np.ones(100), rtol=1e-6)
        assert np.allclose(D, D.T, rtol=1e-7)


def test_diagonal_not_rescaled(small):
    N, rp, ci = small
    S = oracle.sample_uniform(N, 50, 4, 4)
    rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, None, 0, 1)
    deg = np.diff(rp)
    for i, v in enumerate(S):
        row = ciS[rpS[i]:rpS[i + 1]]
        k = rpS[i] + int(np.where(row == i)[0][0])
        assert vS[k] == np.float32(1.0 / deg[v])


def test_against_algorithm2_walkthrough(small):
    N, rp, ci = small
    deg = np.diff(rp).astype(np.float64)
    val = (1.0 / np.sqrt(deg[np.repeat(np.arange(N), np.diff(rp))] * deg[ci])).astype(np.float32)
    for B in (1, 33, 200):
        S = oracle.sample_uniform(N, B, 8, B)
        rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, val, 0, 1)
        rp2, ci2, v2 = algorithm2_literal(N, rp, ci, val, S, 1)
        assert np.array_equal(rpS, rp2) and np.array_equal(ciS, ci2)
        assert np.allclose(vS, v2, rtol=1e-6)


def test_unbiasedness_by_exact_enumeration():
    # Eq. 25: averaged over every B-subset that contains v, the rescaled aggregate equals the
    # full-graph aggregate.  Exact rational arithmetic on the weights' squares is not possible
    # (square roots), so weights are passed in as small rationals stored exactly in fp32.
    N, B = 8, 3
    g = si.graph_from_edges(N, [(0, 1), (0, 2), (0, 3), (1, 2), (3, 4), (4, 5), (5, 6), (6, 7), (2, 7), (0, 7)])
    rp, ci = _np_graph(g)
    rng = np.random.default_rng(0)
    val = (rng.integers(1, 64, len(ci)) / 64.0).astype(np.float32)       # exact in fp32
    x = rng.integers(-8, 9, N)
    p = Fraction(B - 1, N - 1)
    for v in range(N):
        full = sum(Fraction(float(val[e])) * int(x[ci[e]]) for e in range(rp[v], rp[v + 1]))
        subsets = [s for s in itertools.combinations(range(N), B) if v in s]
        tot = Fraction(0)
        for s in subsets:
            S = np.array(s, np.int32)
            rpS, ciS, _ = oracle.induced_csr(N, rp, ci, S, val, 0, 0)
            i = s.index(v)
            for e in range(rpS[i], rpS[i + 1]):
                u = s[ciS[e]]
                a = Fraction(float(val[rp[v] + int(np.where(ci[rp[v]:rp[v + 1]] == u)[0][0])]))
                tot += (a if u == v else a / p) * int(x[u])
        assert tot / len(subsets) == full
    # and the oracle's own rescaled values reproduce it in floating point
    for v in range(N):
        full = sum(float(val[e]) * x[ci[e]] for e in range(rp[v], rp[v + 1]))
        acc, cnt = 0.0, 0
        for s in itertools.combinations(range(N), B):
            if v not in s:
                continue
            S = np.array(s, np.int32)
            rpS, ciS, vS = oracle.induced_csr(N, rp, ci, S, val, 0, 1)
            i = s.index(v)
            acc += sum(float(vS[e]) * x[s[ciS[e]]] for e in range(rpS[i], rpS[i + 1]))
            cnt += 1
        assert abs(acc / cnt - full) < 1e-5


def test_expected_edge_count():
    # E[nnz_S] = B + (E - N) B (B-1) / (N (N-1)) for any graph under Eq. 20
    g = si.rmat_graph(200, 900, seed=5)
    rp, ci = _np_graph(g)
    N, B, T = 200, 40, 600
    tot = 0
    for t in range(T):
        S = oracle.sample_uniform(N, B, 42, t)
        rpS, _, _ = oracle.induced_csr(N, rp, ci, S)
        tot += int(rpS[-1])
    expect = B + (len(ci) - N) * B * (B - 1) / (N * (N - 1))
    assert abs(tot / T - expect) < 0.05 * expect


def test_hand_example():
    # path 0-1-2-3 plus edge 0-3 (a 4-cycle), S = {0,1,3}: N=4, B=3, p = 2/3
    g = si.graph_from_edges(4, [(0, 1), (1, 2), (2, 3), (0, 3)])
    rp, ci = _np_graph(g)
    rpS, ciS, vS = oracle.induced_csr(4, rp, ci, np.array([0, 1, 3], np.int32))
    assert rpS.tolist() == [0, 3, 5, 7]
    assert ciS.tolist() == [0, 1, 2, 0, 1, 0, 2]
    third = 1.0 / 3.0          # every vertex has degree 3 with its self-loop
    exp = [third, third * 1.5, third * 1.5, third * 1.5, third, third * 1.5, third]
    assert np.allclose(vS, exp, rtol=1e-6)


def test_invalid_arguments(small):
    N, rp, ci = small
    with pytest.raises(ValueError):
        oracle.induced_csr(N, rp, ci, np.zeros(0, np.int32))


# ---- Algorithm 2's row / column ranges: one shard of the mini-batch matrix ----

def test_shards_tile_the_full_matrix(tiny_graph):
    g = tiny_graph
    N = g.N; B = 700
    rpg, cig = g.rowptr.numpy(), g.colidx.numpy()
    S = oracle.sample_uniform(N, B, 5, 2)
    rp, ci, v = oracle.induced_csr(N, rpg, cig, S)
    full = csr_to_dense(rp, ci, v, B)
    cuts_r = [0, 1000, 1001, 2500, N]          # ragged, one range of a single vertex
    cuts_c = [0, 17, 3000, N]
    total = np.zeros_like(full); count = 0
    for a, b in zip(cuts_r[:-1], cuts_r[1:]):
        for c, d in zip(cuts_c[:-1], cuts_c[1:]):
            rpt, cit, vt = oracle.induced_csr_range(N, rpg, cig, S, a, b, c, d)
            tile = csr_to_dense(rpt, cit, vt, B)
            # the tile is the full matrix restricted to the rows / columns of S inside the ranges
            rows_in = (S >= a) & (S < b); cols_in = (S >= c) & (S < d)
            want = np.where(rows_in[:, None] & cols_in[None, :], full, 0.0)
            assert np.array_equal(tile, want)
            assert all(np.all(np.diff(cit[rpt[i]:rpt[i + 1]]) > 0) for i in range(B))      # ascending columns
            total += tile; count += len(cit)
    assert np.array_equal(total, full) and count == len(ci)


def test_shard_edge_cases(tiny_graph):
    g = tiny_graph
    rpg, cig = g.rowptr.numpy(), g.colidx.numpy()
    S = oracle.sample_uniform(g.N, 300, 1, 0)
    full = oracle.induced_csr(g.N, rpg, cig, S)
    whole = oracle.induced_csr_range(g.N, rpg, cig, S, 0, g.N, 0, g.N)
    assert all(np.array_equal(a, b) for a, b in zip(full, whole))
    rpt, cit, vt = oracle.induced_csr_range(g.N, rpg, cig, S, 10, 10, 0, g.N)          # empty row range
    assert len(cit) == 0 and np.all(rpt == 0)
    with pytest.raises(ValueError):
        oracle.induced_csr_range(g.N, rpg, cig, S, 0, g.N + 1, 0, g.N)
    # the symmetric matrix of an undirected graph: the transpose of tile (R, C) is tile (C, R)
    a = csr_to_dense(*oracle.induced_csr_range(g.N, rpg, cig, S, 0, 2000, 1500, g.N), 300)
    b = csr_to_dense(*oracle.induced_csr_range(g.N, rpg, cig, S, 1500, g.N, 0, 2000), 300)
    assert np.array_equal(a.T, b)
