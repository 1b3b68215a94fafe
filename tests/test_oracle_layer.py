"""Pins for the oracle's layer forward / backward (Eqs. 5-6, layer-backward equations), the
bf16 rounding, the transpose, the loss and the whole step."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
import synth_inputs as si
from helpers import csr_to_dense, dense_induced


@pytest.fixture(scope="module")
def sub():
    g = si.rmat_graph(400, 2500, seed=21)
    rp = g.rowptr.numpy(); ci = g.colidx.numpy()
    S = oracle.sample_uniform(400, 96, 0, 0)
    rpS, ciS, vS = oracle.induced_csr(400, rp, ci, S)
    return 96, rpS, ciS, vS


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_spmm_against_dense_and_scipy(sub):
    B, rp, ci, v = sub
    H = _rand((B, 19), 1)
    ref = csr_to_dense(rp, ci, v, B) @ H
    got = oracle.spmm(rp, ci, v, H)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
    A = sp.csr_matrix((v.astype(np.float64), ci, rp), shape=(B, B))
    assert np.allclose(got, A @ H, rtol=1e-12, atol=1e-13)


def test_spmm_rectangular_and_empty_rows():
    rp = np.array([0, 0, 2, 2, 3], np.int32); ci = np.array([4, 1, 0], np.int32)
    v = np.array([2.0, -1.0, 0.5], np.float32)
    H = _rand((5, 3), 2)
    got = oracle.spmm(rp, ci, v, H)
    assert np.allclose(got, csr_to_dense(rp, ci, v, 5) @ H)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)


def test_transpose_against_scipy(sub):
    B, rp, ci, v = sub
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)
    A = sp.csr_matrix((v, ci, rp), shape=(B, B)).T.tocsr(); A.sort_indices()
    assert np.array_equal(rpT, A.indptr) and np.array_equal(ciT, A.indices) and np.array_equal(vT, A.data)
    # non-symmetric, rectangular
    rp2 = np.array([0, 2, 3], np.int32); ci2 = np.array([0, 2, 1], np.int32); v2 = np.array([1, 2, 3], np.float32)
    r, c, w = oracle.csr_transpose(2, 3, rp2, ci2, v2)
    assert np.array_equal(csr_to_dense(r, c, w, 2), csr_to_dense(rp2, ci2, v2, 3).T)


def test_gemm_against_numpy():
    A = _rand((37, 23), 3); Bm = _rand((23, 11), 4)
    assert np.allclose(oracle.gemm(A, Bm), A @ Bm, rtol=1e-13, atol=1e-13)
    # a transposed-operand mistake would fail on non-square shapes
    assert oracle.gemm(A, Bm).shape == (37, 11)


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("use_bias", [False, True])
def test_layer_forward_against_dense(sub, relu, use_bias):
    B, rp, ci, v = sub
    H = _rand((B, 13), 5); W = _rand((13, 7), 6); b = _rand(7, 7) if use_bias else None
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, b, relu=relu)
    A = csr_to_dense(rp, ci, v, B)
    Z = A @ H @ W + (b if use_bias else 0.0)
    assert np.allclose(T, A @ H, rtol=1e-12, atol=1e-13)
    assert np.allclose(Y, np.maximum(Z, 0) if relu else Z, rtol=1e-12, atol=1e-12)
    # both association orders agree
    assert np.allclose(A @ (H @ W), (A @ H) @ W, rtol=1e-10, atol=1e-12)


def test_layer_special_cases():
    B = 17
    rp = np.arange(B + 1, dtype=np.int32); ci = np.arange(B, dtype=np.int32); v = np.ones(B, np.float32)
    H = _rand((B, 5), 8); W = _rand((5, 4), 9)
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=False)      # A = I: plain GEMM
    assert np.array_equal(T, H) and np.allclose(Y, H @ W, rtol=1e-13)
    g = si.rmat_graph(50, 150, seed=2)
    S = np.arange(50, dtype=np.int32)
    r, c, w = oracle.induced_csr(50, g.rowptr.numpy(), g.colidx.numpy(), S)
    T, Y = oracle.gcn_fwd(r, c, w, _rand((50, 6), 1), np.eye(6), None, relu=False)   # W = I: plain SpMM
    assert np.allclose(T, Y)


def _torch_layer(A, H, W, b, relu):
    Z = A @ H @ W + (b if b is not None else 0.0)
    return torch.relu(Z) if relu else Z


@pytest.mark.parametrize("relu", [False, True])
def test_layer_backward_against_autograd(sub, relu):
    B, rp, ci, v = sub
    H = _rand((B, 9), 10); W = _rand((9, 6), 11); b = _rand(6, 12); R = _rand((B, 6), 13)
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, b, relu=relu)
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)
    dH, dW, db = oracle.gcn_bwd(rpT, ciT, vT, T, W, Y, R, relu=relu)
    A = torch.tensor(csr_to_dense(rp, ci, v, B))
    Ht, Wt, bt = (torch.tensor(x, requires_grad=True) for x in (H, W, b))
    (_torch_layer(A, Ht, Wt, bt, relu) * torch.tensor(R)).sum().backward()
    assert np.allclose(dH, Ht.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dW, Wt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_layer_backward_with_asymmetric_matrix():
    # a non-symmetric A catches a backward pass that forgets the transpose
    rp = np.array([0, 2, 3, 6], np.int32); ci = np.array([0, 2, 0, 0, 1, 2], np.int32)
    v = np.array([0.5, -1.0, 2.0, 0.25, 3.0, 1.5], np.float32)
    H = _rand((3, 4), 1); W = _rand((4, 2), 2); R = _rand((3, 2), 3)
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=False)
    rpT, ciT, vT = oracle.csr_transpose(3, 3, rp, ci, v)
    dH, dW, _ = oracle.gcn_bwd(rpT, ciT, vT, T, W, Y, R, relu=False)
    A = csr_to_dense(rp, ci, v, 3)
    assert np.allclose(dH, A.T @ (R @ W.T)) and np.allclose(dW, (A @ H).T @ R)
    assert not np.allclose(dH, A @ (R @ W.T))


def test_layer_backward_finite_differences(sub):
    B, rp, ci, v = sub
    H = _rand((B, 5), 20); W = _rand((5, 4), 21); b = _rand(4, 22); R = _rand((B, 4), 23)
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)

    def loss(H_, W_, b_):
        return float((oracle.gcn_fwd(rp, ci, v, H_, W_, b_, relu=True)[1] * R).sum())

    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, b, relu=True)
    dH, dW, db = oracle.gcn_bwd(rpT, ciT, vT, T, W, Y, R, relu=True)
    h = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(12):
        i, j = rng.integers(B), rng.integers(5)
        Hp, Hm = H.copy(), H.copy(); Hp[i, j] += h; Hm[i, j] -= h
        assert abs((loss(Hp, W, b) - loss(Hm, W, b)) / (2 * h) - dH[i, j]) < 1e-6
    for k in range(5):
        for j in range(4):
            Wp, Wm = W.copy(), W.copy(); Wp[k, j] += h; Wm[k, j] -= h
            assert abs((loss(H, Wp, b) - loss(H, Wm, b)) / (2 * h) - dW[k, j]) < 1e-5
    for j in range(4):
        bp, bm = b.copy(), b.copy(); bp[j] += h; bm[j] -= h
        assert abs((loss(H, W, bp) - loss(H, W, bm)) / (2 * h) - db[j]) < 1e-5


def test_adjoint_identity_and_bias_as_ones_column(sub):
    B, rp, ci, v = sub
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)
    x = _rand((B, 3), 30); y = _rand((B, 3), 31)
    assert abs((oracle.spmm(rp, ci, v, x) * y).sum() - (x * oracle.spmm(rpT, ciT, vT, y)).sum()) < 1e-10
    # db equals the dW row of a constant-one input column
    H = _rand((B, 4), 32); W = _rand((4, 3), 33); R = _rand((B, 3), 34)
    T = np.concatenate([oracle.spmm(rp, ci, v, H), np.ones((B, 1))], 1)
    W1 = np.concatenate([W, np.zeros((1, 3))], 0)
    Y = T @ W1
    _, dW, db = oracle.gcn_bwd(rpT, ciT, vT, T, W1, Y, R, relu=False, need_dH=False)
    assert np.allclose(dW[-1], db)


def test_relu_gradient_at_zero_is_zero():
    rp = np.array([0, 1], np.int32); ci = np.array([0], np.int32); v = np.ones(1, np.float32)
    H = np.zeros((1, 2)); W = np.ones((2, 2))
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=True)
    dH, dW, db = oracle.gcn_bwd(rp, ci, v, T, W, Y, np.ones((1, 2)), relu=True)
    assert np.all(dH == 0) and np.all(db == 0)


def test_round_bf16_against_torch():
    x = np.concatenate([_rand(2000, 40), _rand(2000, 41) * 1e-20, _rand(2000, 42) * 1e20,
                        [0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38]])
    x32 = x.astype(np.float32)
    ref = torch.tensor(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(x32), ref)


def test_bf16_layer_rounds_gemm_operands(sub):
    B, rp, ci, v = sub
    H = _rand((B, 8), 50); W = _rand((8, 5), 51)
    T, Y = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=False, bf16=True)
    Tr = torch.tensor(T).float().to(torch.bfloat16).double().numpy()
    Wr = torch.tensor(W).float().to(torch.bfloat16).double().numpy()
    assert np.allclose(Y, Tr @ Wr, rtol=1e-12, atol=1e-13)
    _, Y32 = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=False, bf16=False)
    err = np.linalg.norm(Y - Y32) / np.linalg.norm(Y32)
    assert 0 < err < 2e-2
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)
    R = _rand((B, 5), 52)
    dH, dW, db = oracle.gcn_bwd(rpT, ciT, vT, T, W, Y, R, relu=False, bf16=True)
    Rr = torch.tensor(R).float().to(torch.bfloat16).double().numpy()
    assert np.allclose(dW, Tr.T @ Rr, rtol=1e-12, atol=1e-13)
    assert np.allclose(dH, csr_to_dense(rp, ci, v, B).T @ (Rr @ Wr.T), rtol=1e-12, atol=1e-13)
    assert np.allclose(db, R.sum(0))


def test_softmax_xent_against_torch():
    O = _rand((33, 7), 60); y = np.random.default_rng(61).integers(0, 7, 33).astype(np.int32)
    loss, dO = oracle.softmax_xent(O, y)
    Ot = torch.tensor(O, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(Ot, torch.tensor(y, dtype=torch.long))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12 and np.allclose(dO, Ot.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_whole_step_against_autograd(tiny_graph):
    cfg = si.CONFIGS["tiny"]
    g = tiny_graph
    rp = g.rowptr.numpy(); ci = g.colidx.numpy()
    B = 128
    X = si.normal_features(cfg.N, cfg.d_in).numpy(); labels = si.uniform_labels(cfg.N, cfg.classes).numpy()
    weights = [(W.double().numpy(), b.double().numpy()) for W, b in si.layer_weights(cfg)]
    out = oracle.gcn_step(cfg.N, rp, ci, X, labels, weights, B, 0, 0)
    A = torch.tensor(dense_induced(cfg.N, rp, ci, out["S"]))
    assert np.allclose(csr_to_dense(out["rowptr"], out["colidx"], out["val"], B), A.numpy(), rtol=1e-6)
    A = torch.tensor(csr_to_dense(out["rowptr"], out["colidx"], out["val"], B))
    H = torch.tensor(X[out["S"]].astype(np.float64))
    params = [(torch.tensor(W, requires_grad=True), torch.tensor(b, requires_grad=True)) for W, b in weights]
    for l, (W, b) in enumerate(params):
        H = _torch_layer(A, H, W, b, l < len(params) - 1)
    loss = torch.nn.functional.cross_entropy(H, torch.tensor(labels[out["S"]], dtype=torch.long))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-10
    for l, (W, b) in enumerate(params):
        assert np.allclose(out["dW"][l], W.grad.numpy(), rtol=1e-9, atol=1e-13)
        assert np.allclose(out["db"][l], b.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_relu_tie_band_only_acts_inside_the_band():
    # layers_step(relu_ties=..., tie_band=...) replaces the oracle's own ReLU decision only where the
    # pre-activation lies within the band; outside it the supplied mask is ignored, and with a zero band
    # nothing changes at all.
    rng = np.random.default_rng(0)
    Bn = 12
    dense = (rng.random((Bn, Bn)) < 0.4) * rng.random((Bn, Bn)) + np.eye(Bn)
    rp = [0]; ci = []; v = []
    for i in range(Bn):
        nz = np.nonzero(dense[i])[0]
        ci += list(nz); v += list(dense[i, nz].astype(np.float32)); rp.append(len(ci))
    rp, ci, v = np.array(rp, np.int32), np.array(ci, np.int32), np.array(v, np.float32)
    X = rng.standard_normal((Bn, 5)); y = rng.integers(0, 3, Bn).astype(np.int32)
    Ws = [(rng.standard_normal((5, 6)), rng.standard_normal(6) * 0.1), (rng.standard_normal((6, 3)), np.zeros(3))]
    base = oracle.layers_step(rp, ci, v, X, y, Ws)
    flipped = [~base["relu_mask"][0], None]
    same = oracle.layers_step(rp, ci, v, X, y, Ws, relu_ties=flipped, tie_band=0.0)
    assert all(np.array_equal(a, b) for a, b in zip(same["dW"], base["dW"]))
    # a band that covers the smallest |Z| only: exactly that decision flips, and the gradients move
    T0, Z0 = oracle.gcn_fwd(rp, ci, v, X, Ws[0][0], Ws[0][1], relu=False)
    az = np.abs(Z0); k = np.unravel_index(np.argmin(az), az.shape)
    band = (az[k] * 1.0000001) / az.max()
    out = oracle.layers_step(rp, ci, v, X, y, Ws, relu_ties=flipped, tie_band=band)
    assert out["relu_band"][0].sum() == 1 and out["relu_band"][0][k]
    diff = out["relu_mask"][0] != base["relu_mask"][0]
    assert diff.sum() == 1 and diff[k]
    assert np.array_equal(out["loss"], base["loss"]) and all(np.array_equal(a, b) for a, b in zip(out["H"], base["H"]))
    assert not np.array_equal(out["dW"][0], base["dW"][0])


def _small_stack(rng, Bn=10, scale=1.0):
    dense = (rng.random((Bn, Bn)) < 0.4) * rng.random((Bn, Bn)) + np.eye(Bn)
    rp = [0]; ci = []; v = []
    for i in range(Bn):
        nz = np.nonzero(dense[i])[0]
        ci += list(nz); v += list(dense[i, nz].astype(np.float32)); rp.append(len(ci))
    rp, ci, v = np.array(rp, np.int32), np.array(ci, np.int32), np.array(v, np.float32)
    X = rng.standard_normal((Bn, 4)) * scale; y = rng.integers(0, 3, Bn).astype(np.int32)
    Ws = [(rng.standard_normal((4, 5)), rng.standard_normal(5) * 0.1), (rng.standard_normal((5, 3)), np.zeros(3))]
    return rp, ci, v, X, y, Ws


def test_undecidable_loss_rows_are_the_large_unsaturated_ones():
    # closed cases of the criterion max_j min(p_j, 1-p_j) (e^(2 eps) - 1) > band * max_ij|p - onehot|, eps = band * max|o|:
    # small logits are decidable whatever their gap; large logits with one dominant class are decidable;
    # large logits with two close leaders are not.
    O = np.array([[0.10, 0.09, -0.2],        # small: eps = 2e-3, bound 0.5 * 4e-3
                  [400.0, 100.0, -50.0],      # saturated: 1 - p = e^-300
                  [400.0, 399.5, -50.0],      # two leaders half a unit apart with eps = 8: undecidable
                  [400.0, 360.0, 0.0],        # gap 40 against 2 eps = 16: 1 - p = e^-40, bound e^-24
                  [400.0, 390.0, 0.0]])       # gap 10 < 2 eps: a permitted perturbation swaps the leaders
    y = np.array([2, 1, 0, 0, 0], np.int32)
    assert oracle.undecidable_loss_rows(O, y, 2e-2).tolist() == [False, False, True, False, True]
    assert not oracle.undecidable_loss_rows(O, y, 0.0).any()
    # the bound it is built on holds for every permitted perturbation: rows declared decidable move by less
    # than the band, and some undecidable row moves by far more
    rng = np.random.default_rng(3)
    band = 2e-2
    O = rng.standard_normal((300, 6)) * rng.choice([0.1, 1.0, 30.0, 300.0], (300, 1))
    y = rng.integers(0, 6, 300).astype(np.int32)
    und = oracle.undecidable_loss_rows(O, y, band)
    assert und.any() and not und.all()
    _, g0 = oracle.softmax_xent(O, y)
    eps = band * np.abs(O).max(axis=1, keepdims=True)
    worst = np.zeros(300)
    for _ in range(30):
        _, g1 = oracle.softmax_xent(O + eps * rng.choice([-1.0, 1.0], O.shape), y)
        worst = np.maximum(worst, np.abs(g1 - g0).max(axis=1) / np.abs(g0).max())
    assert worst[~und].max() <= band and worst[und].max() > 5 * band
    # a separate bar for the gradient: logits known four times better than the bar they are measured against
    und4 = oracle.undecidable_loss_rows(O, y, band / 4, band)
    assert und4.sum() < und.sum() and not (und4 & ~und).any()
    worst4 = np.zeros(300)
    for _ in range(30):
        _, g1 = oracle.softmax_xent(O + 0.25 * eps * rng.choice([-1.0, 1.0], O.shape), y)
        worst4 = np.maximum(worst4, np.abs(g1 - g0).max(axis=1) / np.abs(g0).max())
    assert worst4[~und4].max() <= band


def test_loss_gradient_ties_enter_only_inside_the_band():
    # like relu_ties: rows handed in replace the oracle's own loss-gradient rows inside the undecidable set and
    # nowhere else; forward values, loss and the returned dO stay the oracle's own
    rng = np.random.default_rng(1)
    rp, ci, v, X, y, Ws = _small_stack(rng, scale=0.3)      # logits up to about 10: two of the ten rows fall in the band
    base = oracle.layers_step(rp, ci, v, X, y, Ws, logit_band=2e-2)
    loss, dO = oracle.softmax_xent(base["H"][-1], y)
    assert np.array_equal(base["dO"], dO) and base["loss"] == loss
    bandrows = base["dO_band"]
    assert np.array_equal(bandrows, oracle.undecidable_loss_rows(base["H"][-1], y, 2e-2))
    assert bandrows.any() and not bandrows.all()
    ties = rng.standard_normal(dO.shape)           # arbitrary rows: only those inside the band may show
    out = oracle.layers_step(rp, ci, v, X, y, Ws, logit_band=2e-2, dO_ties=ties)
    patched = dO.copy(); patched[bandrows] = ties[bandrows]
    # the weight gradient of the last layer is T^T dO with the patched start
    assert np.allclose(out["dW"][1], base["T"][1].T @ patched, rtol=1e-12, atol=1e-12)
    assert np.allclose(out["db"][1], patched.sum(axis=0), rtol=1e-12, atol=1e-15)
    assert out["loss"] == base["loss"] and np.array_equal(out["dO"], dO)
    assert all(np.array_equal(a, b) for a, b in zip(out["H"], base["H"]))
    # without a band nothing handed in is used
    same = oracle.layers_step(rp, ci, v, X, y, Ws, dO_ties=ties)
    for l in range(2):
        assert np.array_equal(same["dW"][l], oracle.layers_step(rp, ci, v, X, y, Ws)["dW"][l])


def test_stored_bf16_activations_round_once_after_the_activation():
    rng = np.random.default_rng(5)
    rp, ci, v, X, y, Ws = _small_stack(rng)
    full = oracle.layers_step(rp, ci, v, X, y, Ws, bf16=True)
    st = oracle.layers_step(rp, ci, v, X, y, Ws, bf16=True, store_bf16=True)
    # the first layer sees the same input: its stored output is the rounded one, the mask is untouched
    assert np.array_equal(st["H"][1], oracle.round_bf16(full["H"][1])) and not np.array_equal(st["H"][1], full["H"][1])
    assert np.array_equal(st["relu_mask"][0], full["relu_mask"][0])
    assert np.array_equal(st["H"][1], np.asarray(torch.tensor(full["H"][1]).to(torch.bfloat16).double()))
    # the logits are computed from the stored activations and are not rounded themselves
    T2, Z2 = oracle.gcn_fwd(rp, ci, v, st["H"][1], Ws[1][0], Ws[1][1], relu=False, bf16=True)
    assert np.array_equal(st["H"][2], Z2) and np.array_equal(st["T"][1], T2)
    # the gradient handed down to the first layer is stored rounded: its bias gradient is the column sum of the rounded,
    # masked values, and its weight gradient (whose product rounds that operand anyway) is what it would be without storage
    dZ0 = oracle.round_bf16(st["dH"][1]) * st["relu_mask"][0]
    assert np.allclose(st["db"][0], dZ0.sum(axis=0), rtol=1e-13, atol=1e-15)
    assert not np.allclose(st["db"][0], (st["dH"][1] * st["relu_mask"][0]).sum(axis=0), rtol=1e-9, atol=0)
    assert np.allclose(st["dW"][0], oracle.round_bf16(st["T"][0]).T @ dZ0, rtol=1e-12, atol=1e-15)


def test_stored_bf16_gradient_of_the_aggregate_rounds_once_before_the_sparse_product():
    # with stored bfloat16 activations the gradient of the aggregate, dT = dZ W^T, is stored as bfloat16 too: the
    # transposed sparse product reads the rounded values, and nothing else in the layer changes
    import scipy.sparse as sp
    rng = np.random.default_rng(6)
    rp, ci, v, X, y, Ws = _small_stack(rng)
    Bn = len(rp) - 1
    A = sp.csr_matrix((np.asarray(v, np.float64), ci, rp), shape=(Bn, Bn))
    st = oracle.layers_step(rp, ci, v, X, y, Ws, bf16=True, store_bf16=True)
    dZ1 = oracle.round_bf16(st["dO"])                       # operand of the dense product (no ReLU on the last layer)
    dT1_exact = dZ1 @ oracle.round_bf16(Ws[1][0]).T
    dT1 = oracle.round_bf16(dT1_exact)
    assert np.allclose(st["dH"][1], A.T @ dT1, rtol=1e-12, atol=1e-15)
    assert not np.allclose(st["dH"][1], A.T @ dT1_exact, rtol=1e-9, atol=0)
    # the layer function alone: the flag changes dH only, and without it dT stays unrounded
    Ymask = np.ones_like(st["dO"])
    rpT, ciT, vT = oracle.csr_transpose(Bn, Bn, rp, ci, v)
    dH_r, dW_r, db_r = oracle.gcn_bwd(rpT, ciT, vT, st["T"][1], Ws[1][0], Ymask, st["dO"], relu=False, bf16=True, store_dT_bf16=True)
    dH_u, dW_u, db_u = oracle.gcn_bwd(rpT, ciT, vT, st["T"][1], Ws[1][0], Ymask, st["dO"], relu=False, bf16=True)
    assert np.array_equal(dW_r, dW_u) and np.array_equal(db_r, db_u)
    assert np.allclose(dH_u, A.T @ dT1_exact, rtol=1e-12, atol=1e-15) and np.allclose(dH_r, A.T @ dT1, rtol=1e-12, atol=1e-15)


def test_stored_bf16_loss_gradient_changes_the_last_bias_gradient_only():
    # dO stored as bfloat16: the last layer's bias gradient is the column sum of the rounded values; its weight
    # gradient, whose product rounds dO anyway, is what it was; the returned dO is the unrounded one
    rng = np.random.default_rng(7)
    rp, ci, v, X, y, Ws = _small_stack(rng)
    plain = oracle.layers_step(rp, ci, v, X, y, Ws, bf16=True)
    st = oracle.layers_step(rp, ci, v, X, y, Ws, bf16=True, store_bf16=True)
    _, dO = oracle.softmax_xent(st["H"][-1], y)
    assert np.array_equal(st["dO"], dO)
    r = oracle.round_bf16(dO)
    assert np.allclose(st["db"][1], r.sum(axis=0), rtol=1e-13, atol=1e-16)
    assert not np.allclose(st["db"][1], dO.sum(axis=0), rtol=1e-9, atol=0) or np.array_equal(r, dO)
    assert np.allclose(st["dW"][1], oracle.round_bf16(st["T"][1]).T @ r, rtol=1e-12, atol=1e-16)
    # without stored activations the bias gradient sums the unrounded values
    _, dO_p = oracle.softmax_xent(plain["H"][-1], y)
    assert np.allclose(plain["db"][1], dO_p.sum(axis=0), rtol=1e-13, atol=1e-16)
