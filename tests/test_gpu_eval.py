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
