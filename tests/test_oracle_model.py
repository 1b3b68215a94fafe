"""Pins of the oracle's parameter updates and of the complete model step (Fig. 2 of the paper; Sec. III-B,
III-C): the optimizers against torch.optim, the model's loss and every parameter gradient against torch
autograd on a small dense copy of the same mini-batch."""
import numpy as np
import pytest
import torch

import oracle
from helpers import csr_to_dense


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_sgd_against_torch():
    w = _rand(50, 1); gs = [_rand(50, 10 + i) for i in range(5)]
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([wt], lr=0.05, weight_decay=0.01)
    wo = w.copy()
    for g in gs:
        wt.grad = torch.tensor(g); opt.step()
        wo = oracle.sgd_step(wo, g, 0.05, 0.01)
    assert np.allclose(wo, wt.detach().numpy(), rtol=1e-13, atol=0)


def test_adam_against_torch_and_first_step_closed_form():
    w = _rand(64, 2); gs = [_rand(64, 20 + i) for i in range(7)]
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([wt], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    wo, m, v = w.copy(), np.zeros(64), np.zeros(64)
    for t, g in enumerate(gs, 1):
        wt.grad = torch.tensor(g); opt.step()
        wo, m, v = oracle.adam_step(wo, g, m, v, 0.01, t)
        assert np.allclose(wo, wt.detach().numpy(), rtol=1e-12, atol=1e-15), t
    # first step: mhat = g, vhat = g^2, so the step is lr * g / (|g| + eps) = lr * sign(g) up to eps
    w1, _, _ = oracle.adam_step(w, gs[0], np.zeros(64), np.zeros(64), 0.01, 1)
    assert np.allclose(w1 - w, -0.01 * np.sign(gs[0]), rtol=0, atol=1e-8)


def _tiny_batch():
    rng = np.random.default_rng(5)
    Bn = 14
    dense = (rng.random((Bn, Bn)) < 0.3) * rng.random((Bn, Bn))
    dense = dense + np.diag(rng.random(Bn) + 0.5)           # not symmetric: the backward must use the transpose
    rp = [0]; ci = []; v = []
    for i in range(Bn):
        for j in range(Bn):
            if dense[i, j] != 0:
                ci.append(j); v.append(np.float32(dense[i, j]))
        rp.append(len(ci))
    return Bn, np.array(rp, np.int32), np.array(ci, np.int32), np.array(v, np.float32)


@pytest.mark.parametrize("q", [0.0, 0.3])
def test_model_step_against_torch_autograd(q):
    Bn, rp, ci, v = _tiny_batch()
    d_in, d_h, c, L = 5, 8, 3, 3
    X = _rand((Bn, d_in), 1); y = np.random.default_rng(2).integers(0, c, Bn).astype(np.int32)
    params = {"W_in": _rand((d_in, d_h), 3) * 0.5,
              "layers": [(_rand((d_h, d_h), 10 + l) * 0.4, 1.0 + 0.3 * _rand(d_h, 20 + l)) for l in range(L)],
              "W_out": _rand((d_h, c), 4) * 0.5}
    eps, seed, step = 1e-3, 77, 5
    out = oracle.model_step(rp, ci, v, X, y, params, drop_q=q, drop_seed=seed, step=step, eps=eps)
    # the same model with torch, dense A, the oracle's own dropout masks as constants
    A = torch.tensor(csr_to_dense(rp, ci, v, Bn), dtype=torch.float64)
    tp = {"W_in": torch.tensor(params["W_in"], requires_grad=True), "W_out": torch.tensor(params["W_out"], requires_grad=True),
          "layers": [(torch.tensor(W, requires_grad=True), torch.tensor(g, requires_grad=True)) for W, g in params["layers"]]}
    Xh = torch.tensor(X) @ tp["W_in"]
    for l, (W, g) in enumerate(tp["layers"]):
        Z = (A @ Xh) @ W
        n = g * Z / torch.sqrt((Z * Z).mean(dim=1, keepdim=True) + eps)
        keep = oracle.dropout_keep(seed, l, step, Bn * d_h, q).reshape(Bn, d_h) if q > 0 else np.ones((Bn, d_h), bool)
        Xh = torch.relu(n) * torch.tensor(keep / (1 - q)) + Xh
    O = Xh @ tp["W_out"]
    loss = torch.nn.functional.cross_entropy(O, torch.tensor(y, dtype=torch.long))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12
    assert np.allclose(out["O"], O.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(out["dW_in"], tp["W_in"].grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(out["dW_out"], tp["W_out"].grad.numpy(), rtol=1e-10, atol=1e-13)
    for l in range(L):
        assert np.allclose(out["dW"][l], tp["layers"][l][0].grad.numpy(), rtol=1e-10, atol=1e-13), l
        assert np.allclose(out["dgamma"][l], tp["layers"][l][1].grad.numpy(), rtol=1e-10, atol=1e-13), l


def test_binary_cross_entropy_against_torch_and_closed_forms():
    O = _rand((17, 9), 40) * 4; Y = (np.random.default_rng(41).random((17, 9)) < 0.3).astype(np.float64)
    loss, dO = oracle.sigmoid_bce(O, Y)
    ot = torch.tensor(O, requires_grad=True)
    lt = torch.nn.functional.binary_cross_entropy_with_logits(ot, torch.tensor(Y))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-13 and np.allclose(dO, ot.grad.numpy(), rtol=1e-12, atol=1e-16)
    # zero logits: every entry costs log 2; saturated logits of the right sign cost nothing and stay finite
    l0, d0 = oracle.sigmoid_bce(np.zeros((3, 4)), Y[:3, :4])
    assert abs(l0 - np.log(2.0)) < 1e-15 and np.allclose(d0, (0.5 - Y[:3, :4]) / 12)
    big = np.where(Y > 0, 800.0, -800.0)
    lb, db = oracle.sigmoid_bce(big, Y)
    assert lb == 0.0 and np.all(db == 0.0)
    lw, _ = oracle.sigmoid_bce(-big, Y)
    assert abs(lw - 800.0) < 1e-9
