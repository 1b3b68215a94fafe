"""Pins of the oracle's layer tail (Sec. III-B Eqs. 7-10: RMSNorm, ReLU, dropout, residual add; Sec. III-C
element-wise backward) against what the mathematics fixes: closed forms, invariants, an independent
re-evaluation of the dropout counter mapping, torch autograd and central finite differences."""
import numpy as np
import pytest
import torch

import oracle
from helpers import philox_py


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_rmsnorm_closed_form_small():
    # x = (3, 4): mean square 12.5, rms = sqrt(12.5)
    Y, ir, Xn = oracle.tail_fwd(np.array([[3.0, 4.0]]), eps=0.0)
    r = np.sqrt(12.5)
    assert np.allclose(ir, [1 / r], rtol=0, atol=1e-15)
    assert np.allclose(Xn, [[3 / r, 4 / r]], rtol=0, atol=1e-15)
    assert np.allclose(Y, Xn)          # both positive: ReLU keeps them, no dropout, no residual


def test_rmsnorm_rows_have_unit_rms_and_scale_invariance():
    Z = _rand((37, 50), 1) * np.exp(_rand((37, 1), 2) * 3)       # rows of very different magnitude
    _, ir, Xn = oracle.tail_fwd(Z, eps=0.0)
    assert np.allclose(np.sqrt((Xn ** 2).mean(axis=1)), 1.0, rtol=1e-13)
    _, _, Xn2 = oracle.tail_fwd(Z * 7.5, eps=0.0)
    assert np.allclose(Xn, Xn2, rtol=1e-13, atol=0)                # RMSNorm(c x) = RMSNorm(x), c > 0
    _, _, Xn3 = oracle.tail_fwd(-Z, eps=0.0)
    assert np.allclose(Xn3, -Xn, rtol=1e-13, atol=0)               # odd


def test_rmsnorm_scale_and_eps():
    Z = _rand((9, 16), 3); g = _rand(16, 4)
    _, ir, Xn = oracle.tail_fwd(Z, gamma=g, eps=0.25)
    want_ir = 1.0 / np.sqrt((Z ** 2).mean(axis=1) + 0.25)
    assert np.allclose(ir, want_ir, rtol=1e-14)
    assert np.allclose(Xn, Z * want_ir[:, None] * g[None, :], rtol=1e-13)
    # a zero row is finite with eps > 0
    Y, ir0, _ = oracle.tail_fwd(np.zeros((1, 8)), eps=1e-6)
    assert np.all(Y == 0) and np.isfinite(ir0).all()


def test_relu_and_residual():
    Z = _rand((20, 12), 5); R = _rand((20, 12), 6)
    Y0, _, Xn = oracle.tail_fwd(Z, eps=0.0)
    assert np.array_equal(Y0, np.maximum(Xn, 0))
    Y1, _, _ = oracle.tail_fwd(Z, eps=0.0, R=R)
    assert np.allclose(Y1 - Y0, R, rtol=0, atol=1e-15)


def test_dropout_mask_follows_the_counter_mapping():
    # independent evaluation of the pinned definition with the big-integer Philox of tests/helpers.py
    seed, layer, step, q = 0x1234567890ABCDEF, 3, 11, 0.3
    keep = oracle.dropout_keep(seed, layer, step, 41, q)
    thr = int(np.floor(q * 2 ** 32))
    for e in range(41):
        blk = e // 4
        out = philox_py([blk & 0xFFFFFFFF, blk >> 32, step, 0x80000000 + layer], [seed & 0xFFFFFFFF, seed >> 32])
        assert keep[e] == (out[e % 4] >= thr)


def test_dropout_statistics_scaling_and_determinism():
    q = 0.25
    n = 200000
    keep = oracle.dropout_keep(7, 0, 0, n, q)
    frac = keep.mean()
    assert abs(frac - (1 - q)) < 5 * np.sqrt(q * (1 - q) / n)
    assert np.array_equal(keep, oracle.dropout_keep(7, 0, 0, n, q))
    for other in (oracle.dropout_keep(8, 0, 0, n, q), oracle.dropout_keep(7, 1, 0, n, q), oracle.dropout_keep(7, 0, 1, n, q)):
        agree = (other == keep).mean()            # independent masks agree with probability q^2 + (1-q)^2
        assert abs(agree - (q * q + (1 - q) ** 2)) < 0.01
    # q = 0 keeps everything; the mask does not depend on the values; kept values are scaled by 1 / (1 - q)
    assert oracle.dropout_keep(7, 0, 0, 1000, 0.0).all()
    Z = np.abs(_rand((50, 40), 8)) + 0.1
    Yq, _, Xn = oracle.tail_fwd(Z, eps=0.0, q=q, seed=7)
    k = oracle.dropout_keep(7, 0, 0, Z.size, q).reshape(Z.shape)
    assert np.allclose(Yq, np.where(k, Xn / (1 - q), 0.0), rtol=1e-14)
    # nested thresholds: whatever survives a higher drop rate survives a lower one
    assert np.all(oracle.dropout_keep(7, 0, 0, 5000, 0.1)[oracle.dropout_keep(7, 0, 0, 5000, 0.6)])


@pytest.mark.parametrize("q", [0.0, 0.4])
@pytest.mark.parametrize("with_gamma", [False, True])
def test_backward_against_torch_autograd(q, with_gamma):
    Bn, d = 23, 31
    Z = _rand((Bn, d), 10); dY = _rand((Bn, d), 11); g = _rand(d, 12) if with_gamma else None
    eps = 1e-3
    dZ, dg = oracle.tail_bwd(Z, dY, gamma=g, eps=eps, q=q, seed=5, layer=2, step=9)
    keep = oracle.dropout_keep(5, 2, 9, Bn * d, q).reshape(Bn, d) if q > 0 else np.ones((Bn, d), bool)
    zt = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(g if g is not None else np.ones(d), dtype=torch.float64, requires_grad=True)
    n = gt * zt / torch.sqrt((zt * zt).mean(dim=1, keepdim=True) + eps)
    y = torch.relu(n) * torch.tensor(keep / (1 - q) if q > 0 else keep.astype(float))
    y.backward(torch.tensor(dY))
    assert np.allclose(dZ, zt.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(dg, gt.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_backward_against_central_differences():
    Bn, d = 4, 6
    Z = _rand((Bn, d), 20); dY = _rand((Bn, d), 21); g = _rand(d, 22); R = _rand((Bn, d), 23)
    kw = dict(eps=1e-2, q=0.3, seed=3, layer=1, step=4)
    dZ, dg = oracle.tail_bwd(Z, dY, gamma=g, **kw)
    _, _, Xn = oracle.tail_fwd(Z, gamma=g, R=R, **kw)
    assert np.abs(Xn).min() > 1e-3          # no element sits at the ReLU kink
    f = lambda Zv, gv: float((oracle.tail_fwd(Zv, gamma=gv, R=R, **kw)[0] * dY).sum())
    h = 1e-6
    for i in range(Bn):
        for j in range(d):
            Zp = Z.copy(); Zp[i, j] += h; Zm = Z.copy(); Zm[i, j] -= h
            assert abs((f(Zp, g) - f(Zm, g)) / (2 * h) - dZ[i, j]) < 1e-6 * max(1.0, abs(dZ[i, j]))
    for j in range(d):
        gp = g.copy(); gp[j] += h; gm = g.copy(); gm[j] -= h
        assert abs((f(Z, gp) - f(Z, gm)) / (2 * h) - dg[j]) < 1e-6 * max(1.0, abs(dg[j]))


def test_backward_is_orthogonal_to_the_row_direction():
    # RMSNorm is invariant to a positive rescale of a row (eps = 0), so the gradient has no component along z
    Z = _rand((15, 20), 30); dY = _rand((15, 20), 31); g = _rand(20, 32)
    dZ, _ = oracle.tail_bwd(Z, dY, gamma=g, eps=0.0, q=0.2, seed=1)
    assert np.abs((dZ * Z).sum(axis=1)).max() < 1e-12 * np.abs(dZ).max() * np.abs(Z).max() * 20
