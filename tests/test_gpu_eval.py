"""Full-graph evaluation forward: the GCN layers over all N vertices with the normalised adjacency of Eq. 3
(no sampling, no 1/p rescale) - the paper's evaluation rounds - against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si
from gpu_util import DEV, TOL_F32, TOL_VAL
from helpers import rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i64", [False, True])
def test_full_graph_matrix_and_forward(i64):
    cfg = si.CONFIGS["tiny"]
    g = si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=DEV)
    rowptr = g.rowptr if i64 else g.rowptr.to(torch.int32)
    c = sg.Context(0)
    E = int(g.colidx.numel())
    c.reserve(cfg.N, E, cfg.N, 64, E)
    A = sg.sgnn_graph_normalized_csr(c, cfg.N, rowptr, g.colidx)
    # the oracle's statement of the same matrix: the induced matrix of the whole vertex set (B = N, p = 1)
    rp, ci, v = oracle.induced_csr(cfg.N, g.rowptr.cpu().numpy(), g.colidx.cpu().numpy(), np.arange(cfg.N, dtype=np.int32))
    assert np.array_equal(A.rowptr.cpu().numpy(), rp)
    assert np.array_equal(A.colidx.cpu().numpy(), ci)
    assert rel_err(A.val.cpu().numpy()[:E], v) < TOL_VAL
    # two layers over all vertices
    X = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=DEV)
    weights = si.layer_weights(cfg)
    H = X
    Href = X.cpu().numpy().astype(np.float64)
    for l, (W, b) in enumerate(weights):
        relu = l < len(weights) - 1
        Y = torch.empty((cfg.N, W.shape[1]), dtype=torch.float32, device=DEV)
        T = torch.empty((cfg.N, W.shape[0]), dtype=torch.float32, device=DEV)
        sg.sgnn_gcn_fwd(c, A, H, W.to(DEV), b.to(DEV), sg.SGNN_RELU if relu else 0, Y, T)
        _, Href = oracle.gcn_fwd(rp, ci, v, Href, W.numpy(), b.numpy(), relu=relu)
        assert rel_err(Y.cpu().numpy(), Href) < TOL_F32, l
        H = Y
    c.status()
    c.close()


@pytest.mark.parametrize("d", [32, 128, 256])
def test_sparse_product_with_int64_row_offsets(d):
    """A matrix whose row offsets are int64 (how a full graph with 2^31 entries or more is handed in): the same
    result, bit for bit, as with int32 offsets, with and without a plan; long rows included."""
    rng = np.random.default_rng(5)
    rows, cols = 500, 6000
    lens = rng.integers(0, 6, rows)
    lens[[3, 77, 400]] = [3000, 700, 65]
    lists = [np.sort(rng.choice(cols, n, replace=False)).astype(np.int32) for n in lens]
    rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci = np.concatenate(lists); v = rng.standard_normal(len(ci)).astype(np.float32)
    c = sg.Context(0)
    c.reserve(cols, len(ci), rows, d, len(ci))
    X = torch.tensor(rng.standard_normal((cols, d)).astype(np.float32), device=DEV)
    A32 = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV, with_plan=True)
    sg.sgnn_csr_plan(c, A32)
    ref = torch.zeros((rows, d), dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(c, A32, X, ref)
    assert rel_err(ref.cpu().numpy(), oracle.spmm(rp, ci, v, X.cpu().numpy().astype(np.float64))) < TOL_F32
    for with_plan in (False, True):
        A64 = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV, with_plan=with_plan)
        A64.rowptr = A64.rowptr.to(torch.int64)
        if with_plan:
            sg.sgnn_csr_plan(c, A64)
        out = torch.full((rows, d), 3.0, dtype=torch.float32, device=DEV)
        sg.sgnn_spmm(c, A64, X, out)
        assert torch.equal(out, ref)
    # calls that write or reorder a matrix keep int32 offsets
    AT = sg.Csr(cols, rows, len(ci), DEV)
    with pytest.raises(sg.SgnnError):
        sg.sgnn_csr_transpose(c, A64, AT)
    c.status()
    c.close()
