"""GPU parity: sampler and induced CSR against the CPU oracle, bit-exact on indices."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si
from gpu_util import DEV, TOL_VAL, bitmap_rank_from_sample, ctx, dev, gpu_sample

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,B,seed,step", [
    (1, 1, 0, 0), (2, 1, 0, 0), (63, 17, 1, 2), (64, 64, 0, 0), (65, 64, 3, 1), (129, 1, 0, 5),
    (4096, 1024, 0, 0), (4096, 1024, 0, 1), (5000, 4999, 9, 9), (100003, 777, 2**40 + 3, 2**35 + 1),
    (262144, 32768, 0, 0), (262144, 32768, 0, 15), (1000003, 1000003, 4, 4), (1000003, 250000, 5, 6),
    # from 2^20 vertices on the later passes read stored key prefixes: even and odd N, ragged last quad and last word,
    # B = N, nearly all, a handful
    (1048576, 1000, 1, 1), (1048577, 1048577, 2, 3), (1048583, 5, 3, 0), (2097213, 1048576, 8, 8), (1048583, 1048576, 0, 2),
    (3000001, 300000, 11, 2**33),
    # sparse samples of large graphs take one pass over the keys with a window of histogram bins named in advance:
    # thresholds in the middle of a bin, and expected right on a bin boundary (a window of two bins)
    (4194304, 4096, 6, 1), (8388608, 65536, 7, 2), (2097152, 2000, 1, 9), (4194304, 1, 0, 3),
])
def test_sampler_matches_oracle(N, B, seed, step):
    S, bitmap, rank = gpu_sample(N, B, seed, step)
    S_ref = oracle.sample_uniform(N, B, seed, step)
    assert np.array_equal(S.cpu().numpy(), S_ref)
    words, rk = bitmap_rank_from_sample(N, S_ref)
    assert np.array_equal(bitmap.cpu().numpy(), words)
    assert np.array_equal(rank.cpu().numpy(), rk)


@pytest.mark.parametrize("shift", [-3, 2])
@pytest.mark.parametrize("N,B", [(1048576, 1000), (4194304, 4096)])
def test_sampler_window_that_misses_falls_back(N, B, shift, monkeypatch):
    # With its window of histogram bins moved off its place (a debugging switch of the library, read at every call) the
    # one-pass form of the sampler finds the threshold's bin outside it and the recomputing passes take over; the
    # call after it, with the window in place again, starts from a clean state.
    S_ref = oracle.sample_uniform(N, B, 4, 4)
    monkeypatch.setenv("SGNN_SAMPLER_WINDOW_SHIFT", str(shift))
    S, bitmap, rank = gpu_sample(N, B, 4, 4)
    assert np.array_equal(S.cpu().numpy(), S_ref)
    words, rk = bitmap_rank_from_sample(N, S_ref)
    assert np.array_equal(bitmap.cpu().numpy(), words) and np.array_equal(rank.cpu().numpy(), rk)
    monkeypatch.delenv("SGNN_SAMPLER_WINDOW_SHIFT")
    S, bitmap, rank = gpu_sample(N, B, 4, 4)
    assert np.array_equal(S.cpu().numpy(), S_ref)
    assert np.array_equal(bitmap.cpu().numpy(), words) and np.array_equal(rank.cpu().numpy(), rk)


def test_sampler_is_deterministic_and_stateless():
    a = gpu_sample(300000, 30000, 7, 11)[0].cpu().numpy()
    gpu_sample(4096, 10, 1, 1)
    b = gpu_sample(300000, 30000, 7, 11)[0].cpu().numpy()
    assert np.array_equal(a, b)


def test_sampler_large_n():
    # the vertex count of the largest configuration; B as in that configuration
    N, B = 111059956, 1048576
    S, bitmap, rank = gpu_sample(N, B, 0, 0)
    S_ref = oracle.sample_uniform(N, B, 0, 0)
    assert np.array_equal(S.cpu().numpy(), S_ref)
    words, rk = bitmap_rank_from_sample(N, S_ref)
    assert np.array_equal(bitmap.cpu().numpy(), words) and np.array_equal(rank.cpu().numpy(), rk)


def test_sampler_rejects_bad_arguments():
    S = torch.zeros(8, dtype=torch.int32, device=DEV)
    bm = torch.zeros(1, dtype=torch.int64, device=DEV)
    rk = torch.zeros(1, dtype=torch.int32, device=DEV)
    for N, B in [(10, 0), (10, 11)]:
        with pytest.raises(sg.SgnnError) as e:
            sg.lib()  # make sure the library is the one in use
            ctx().check(sg.lib().sgnn_sample_uniform(ctx()._h, N, B, 0, 0, S.data_ptr(), bm.data_ptr(), rk.data_ptr(), None))
        assert e.value.code == -1
    with pytest.raises(sg.SgnnError):
        ctx().check(sg.lib().sgnn_sample_uniform(ctx()._h, 10, 5, 0, 0, None, bm.data_ptr(), rk.data_ptr(), None))
    with pytest.raises(sg.SgnnError):
        ctx().check(sg.lib().sgnn_sample_uniform(ctx()._h, 2**31, 5, 0, 0, S.data_ptr(), bm.data_ptr(), rk.data_ptr(), None))


def _induce_gpu(g, B, seed, step, norm_mode=0, rescale=1, val=None, rowptr_dtype=torch.int64, capacity=None):
    N = g.N
    rowptr = g.rowptr.to(rowptr_dtype).to(DEV)
    colidx = g.colidx.to(DEV)
    ctx().reserve(N, g.E, B, 1, 0)
    S, bitmap, rank = gpu_sample(N, B, seed, step)
    S_ref = oracle.sample_uniform(N, B, seed, step)
    ref = oracle.induced_csr(N, g.rowptr.numpy(), g.colidx.numpy(), S_ref, val, norm_mode, rescale)
    cap = len(ref[1]) if capacity is None else capacity
    out = sg.Csr(B, B, cap, DEV)
    out.rowptr.fill_(-7); out.colidx.fill_(-7)
    vt = None if val is None else dev(val)
    nnz = sg.sgnn_induced_csr(ctx(), N, rowptr, colidx, vt, S, B, bitmap, rank, out, norm_mode, rescale, want_nnz=True)
    ctx().status()
    return out, nnz, ref


def _assert_csr_equal(out, nnz, ref):
    rp, ci, v = ref
    assert nnz == len(ci) == out.nnz()
    assert np.array_equal(out.rowptr.cpu().numpy(), rp)
    assert np.array_equal(out.colidx.cpu().numpy()[:nnz], ci)
    got = out.val.cpu().numpy()[:nnz].astype(np.float64)
    assert np.all(np.abs(got - v) <= TOL_VAL * np.abs(v))


@pytest.mark.parametrize("norm_mode", [0, 1])
@pytest.mark.parametrize("rescale", [0, 1])
@pytest.mark.parametrize("B", [1, 2, 100, 1024, 4096])
def test_induced_tiny(tiny_graph, B, rescale, norm_mode):
    out, nnz, ref = _induce_gpu(tiny_graph, B, 0, B, norm_mode, rescale)
    _assert_csr_equal(out, nnz, ref)


def test_induced_all_vertices_is_identity(tiny_graph):
    g = tiny_graph
    out, nnz, ref = _induce_gpu(g, g.N, 0, 0)
    assert np.array_equal(out.rowptr.cpu().numpy(), g.rowptr.numpy())
    assert np.array_equal(out.colidx.cpu().numpy()[:nnz], g.colidx.numpy())
    _assert_csr_equal(out, nnz, ref)


def test_induced_int32_rowptr_and_given_weights(tiny_graph):
    g = tiny_graph
    rng = np.random.default_rng(3)
    val = rng.random(g.E).astype(np.float32) + 0.5
    out, nnz, ref = _induce_gpu(g, 700, 1, 2, 0, 1, val=val, rowptr_dtype=torch.int32)
    _assert_csr_equal(out, nnz, ref)


@pytest.fixture(scope="module")
def medium_graph():
    cfg = si.CONFIGS["medium"]
    return si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed)


@pytest.mark.parametrize("step", [0, 7, 15])
def test_induced_medium(medium_graph, step):
    cfg = si.CONFIGS["medium"]
    out, nnz, ref = _induce_gpu(medium_graph, cfg.B, cfg.sampler_seed, step)
    _assert_csr_equal(out, nnz, ref)


def test_induced_medium_ragged_sizes(medium_graph):
    # B not a multiple of anything, hub rows split across many tiles
    out, nnz, ref = _induce_gpu(medium_graph, 100001, 3, 1)
    _assert_csr_equal(out, nnz, ref)
    out, nnz, ref = _induce_gpu(medium_graph, 2049, 3, 2, norm_mode=1)
    _assert_csr_equal(out, nnz, ref)


def test_induced_graph_with_empty_rows():
    # rows without any stored entry (not canonical, but the extraction must still be exact)
    N = 300
    rng = np.random.default_rng(1)
    rows = []
    for v in range(N):
        if v % 3 == 0 or v > 280:
            rows.append(np.zeros(0, np.int32))
        else:
            rows.append(np.unique(rng.integers(0, N, rng.integers(1, 40))).astype(np.int32))
    rowptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int64)
    colidx = np.concatenate(rows).astype(np.int32)
    g = si.Graph(N, torch.as_tensor(rowptr), torch.as_tensor(colidx))
    val = np.ones(len(colidx), np.float32)
    for B in (50, 299, 300):
        out, nnz, ref = _induce_gpu(g, B, 5, B, 0, 1, val=val)
        _assert_csr_equal(out, nnz, ref)


def test_induced_sparse_sample_of_a_large_graph():
    # 17 M vertices, a sample of under 1/32 of them: the extraction screens the edges with its coarse filter (one bit
    # per eight vertices) before it probes the bitmap; result bit for bit as always.  A few sampled vertices are given
    # all-sampled neighbourhoods by construction of the check below: every stored entry is compared.
    N, B = (1 << 24) + 1234567, 300_001
    g = si.rmat_graph(N, 12_000_000, 77, device=DEV)
    rowptr, colidx = g.rowptr, g.colidx
    ctx().reserve(N, g.E, B, 1, 0)
    S, bitmap, rank = gpu_sample(N, B, 3, 5)
    S_ref = oracle.sample_uniform(N, B, 3, 5)
    assert np.array_equal(S.cpu().numpy(), S_ref)
    rp, ci, v = oracle.induced_csr(N, rowptr.cpu().numpy(), colidx.cpu().numpy(), S_ref)
    assert len(ci) > B          # some off-diagonal entries survive
    out = sg.Csr(B, B, len(ci), DEV)
    nnz = sg.sgnn_induced_csr(ctx(), N, rowptr, colidx, None, S, B, bitmap, rank, out, want_nnz=True)
    ctx().status()
    assert nnz == len(ci)
    assert np.array_equal(out.rowptr.cpu().numpy(), rp) and np.array_equal(out.colidx.cpu().numpy()[:nnz], ci)
    got = out.val.cpu().numpy()[:nnz].astype(np.float64)
    assert np.all(np.abs(got - v) <= TOL_VAL * np.abs(v))


def test_induced_dense_rows_of_a_small_graph():
    # 20000 vertices with 1000 entries a row, half of them sampled: the bitmap is small and the tiles are many, which is
    # where the count pass probes a copy of the bitmap in LDS; result bit for bit as always.
    N, B = 20000, 10000
    g = si.rmat_graph(N, 10_000_000, 5, device=DEV)
    assert g.E * B // N // 2048 >= 4096
    ctx().reserve(N, g.E, B, 1, 0)
    S, bitmap, rank = gpu_sample(N, B, 1, 2)
    S_ref = oracle.sample_uniform(N, B, 1, 2)
    rp, ci, v = oracle.induced_csr(N, g.rowptr.cpu().numpy(), g.colidx.cpu().numpy(), S_ref)
    out = sg.Csr(B, B, len(ci), DEV)
    nnz = sg.sgnn_induced_csr(ctx(), N, g.rowptr, g.colidx, None, S, B, bitmap, rank, out, want_nnz=True)
    ctx().status()
    _assert_csr_equal(out, nnz, (rp, ci, v))


def test_induced_capacity_of_half_the_entries(tiny_graph):
    # Capacity for half the entries of a matrix of many tiles: the row offsets are complete, every entry below the
    # capacity is written as usual, none beyond it, and the status word reports the overflow.
    g = tiny_graph
    N, B = g.N, g.N
    ref = oracle.induced_csr(N, g.rowptr.numpy(), g.colidx.numpy(), oracle.sample_uniform(N, B, 0, 0))
    cap = len(ref[1]) // 2
    assert cap > 3 * 2048
    S, bitmap, rank = gpu_sample(N, B, 0, 0)
    out = sg.Csr(B, B, cap, DEV)
    sg.sgnn_induced_csr(ctx(), N, g.rowptr.to(DEV), g.colidx.to(DEV), None, S, B, bitmap, rank, out)
    with pytest.raises(sg.SgnnError) as e:
        ctx().status()
    assert e.value.code == -2
    assert np.array_equal(out.rowptr.cpu().numpy(), ref[0])
    assert np.array_equal(out.colidx.cpu().numpy()[:cap], ref[1][:cap])
    got = out.val.cpu().numpy()[:cap].astype(np.float64)
    assert np.all(np.abs(got - ref[2][:cap]) <= TOL_VAL * np.abs(ref[2][:cap]))


@pytest.mark.parametrize("max_entries", [0, 1 << 20])
def test_induced_in_a_context_of_its_own(medium_graph, max_entries):
    # A context of its own, reserved for exactly this graph and sample (with and without room for mini-batch entries in
    # its scratch), gives the same matrix as the shared, generously reserved one of the other tests.
    g = medium_graph
    cfg = si.CONFIGS["medium"]
    N, B = g.N, cfg.B
    c = sg.Context(0)
    c.reserve(N, g.E, B, 1, max_entries)
    S, bitmap, rank = gpu_sample(N, B, cfg.sampler_seed, 3)
    ref = oracle.induced_csr(N, g.rowptr.numpy(), g.colidx.numpy(), oracle.sample_uniform(N, B, cfg.sampler_seed, 3))
    assert len(ref[1]) <= 1 << 20
    out = sg.Csr(B, B, len(ref[1]), DEV)
    nnz = sg.sgnn_induced_csr(c, N, g.rowptr.to(DEV), g.colidx.to(DEV), None, S, B, bitmap, rank, out, want_nnz=True)
    c.status()
    _assert_csr_equal(out, nnz, ref)


def test_induced_capacity_overflow_is_reported(tiny_graph):
    g = tiny_graph
    with pytest.raises(sg.SgnnError) as e:
        _induce_gpu(g, 1024, 0, 0, capacity=100)
    assert e.value.code == -2
    # the row pointer is still complete and the first `capacity` entries are right
    N, B = g.N, 1024
    S, bitmap, rank = gpu_sample(N, B, 0, 0)
    out = sg.Csr(B, B, 100, DEV)
    sg.sgnn_induced_csr(ctx(), N, g.rowptr.to(DEV), g.colidx.to(DEV), None, S, B, bitmap, rank, out)
    ref = oracle.induced_csr(N, g.rowptr.numpy(), g.colidx.numpy(), oracle.sample_uniform(N, B, 0, 0))
    assert np.array_equal(out.rowptr.cpu().numpy(), ref[0])
    assert out.nnz() == len(ref[1])
    assert np.array_equal(out.colidx.cpu().numpy()[:100], ref[1][:100])
    # without a host read-back of the count the overflow is sticky in the device status word: the next status query
    # fails with the capacity code (once), so a training loop on the asynchronous path cannot run on a cut matrix unnoticed
    with pytest.raises(sg.SgnnError) as e:
        ctx().status()
    assert e.value.code == -2 and "capacity" in str(e.value)
    ctx().status()
    # a matrix that fits leaves the word clear
    out = sg.Csr(B, B, len(ref[1]), DEV)
    sg.sgnn_induced_csr(ctx(), N, g.rowptr.to(DEV), g.colidx.to(DEV), None, S, B, bitmap, rank, out)
    ctx().status()
