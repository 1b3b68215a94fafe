"""The complete model (input projection, residual layers with the fused tail, output head, loss, backward,
parameter update; Fig. 2 and Alg. 1 of the paper) on the HIP library against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si
from gpu_util import DEV, TOL_F32, TOL_BF16, ctx
from helpers import rel_err

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def dev(a, dtype=torch.float32):
    return torch.tensor(np.ascontiguousarray(a), dtype=dtype, device=DEV)


def test_spmm_with_addend(tiny_graph):
    g = tiny_graph
    S = oracle.sample_uniform(g.N, 600, 3, 1)
    rp, ci, v = oracle.induced_csr(g.N, g.rowptr.numpy(), g.colidx.numpy(), S)[:3]
    B = len(S)
    ctx().reserve(B, len(ci), B, 64, len(ci))
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    for d in (64, 47):
        X = _rand((B, d), 1); R = _rand((B, d), 2)
        out = torch.zeros((B, d), dtype=torch.float32, device=DEV)
        sg.sgnn_spmm(ctx(), A, dev(X), out, add=dev(R))
        assert rel_err(out.cpu().numpy(), oracle.spmm(rp, ci, v, X) + R) < TOL_F32


def test_optimizer_steps():
    n = 10007
    w = _rand(n, 1); gs = [_rand(n, 10 + i) for i in range(4)]
    wd_ = dev(w); wo = w.astype(np.float64)
    for g in gs:
        sg.sgnn_sgd_step(ctx(), wd_, dev(g), 0.05, 0.01)
        wo = oracle.sgd_step(wo, g, 0.05, 0.01)
    assert rel_err(wd_.cpu().numpy(), wo) < TOL_F32
    wa = dev(w); m = torch.zeros(n, device=DEV); v = torch.zeros(n, device=DEV)
    wo, mo, vo = w.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(gs, 1):
        sg.sgnn_adam_step(ctx(), wa, dev(g), m, v, 0.01, t)
        wo, mo, vo = oracle.adam_step(wo, g, mo, vo, 0.01, t)
    assert rel_err(wa.cpu().numpy(), wo) < TOL_F32
    assert rel_err(m.cpu().numpy(), mo) < TOL_F32 and rel_err(v.cpu().numpy(), vo) < TOL_F32
    with pytest.raises(sg.SgnnError):
        sg.sgnn_adam_step(ctx(), wa, dev(gs[0]), m, v, 0.01, 0)       # steps are numbered from 1


def _model_inputs(d_in=32, d_h=64, c=8, L=2, seed=0):
    cfg = si.CONFIGS["tiny"]
    gd = si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=DEV)
    Xd = si.normal_features(cfg.N, d_in, cfg.feature_seed, device=DEV)
    # a task the model can learn: the label is the largest of c fixed random projections of the vertex's features
    Wtrue = dev(_rand((d_in, c), 99 + seed))
    ld = torch.argmax(Xd @ Wtrue, dim=1).to(torch.int32)
    params = {"W_in": si.glorot_uniform(d_in, d_h, 100 + seed),
              "layers": [(si.glorot_uniform(d_h, d_h, 110 + seed + l), 1.0 + 0.1 * torch.tensor(_rand(d_h, 120 + seed + l)))
                         for l in range(L)],
              "W_out": si.glorot_uniform(d_h, c, 130 + seed)}
    return cfg, gd, Xd, ld, params


def _to_dev(params):
    return {"W_in": params["W_in"].to(DEV).contiguous(), "W_out": params["W_out"].to(DEV).contiguous(),
            "layers": [(W.to(DEV).contiguous(), g.to(DEV).float().contiguous()) for W, g in params["layers"]]}


def _to_np(params):
    return {"W_in": params["W_in"].double().cpu().numpy(), "W_out": params["W_out"].double().cpu().numpy(),
            "layers": [(W.double().cpu().numpy(), g.double().cpu().numpy()) for W, g in params["layers"]]}


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("q", [0.0, 0.2])
def test_model_step_matches_oracle(q, bf16):
    cfg, gd, Xd, ld, params = _model_inputs()
    tol = TOL_BF16 if bf16 else TOL_F32
    mdl = sg.ScaleGnnModel(cfg.N, gd.rowptr, gd.colidx, Xd, ld, _to_dev(params), cfg.B, sampler_seed=cfg.sampler_seed,
                           drop_q=q, drop_seed=5, eps=1e-6, bf16=bf16, optimizer=None, device=DEV)
    t = 3
    mdl.step(t)
    torch.cuda.synchronize(); mdl.ctx.status()
    rpg, cig = gd.rowptr.cpu().numpy(), gd.colidx.cpu().numpy()
    S = oracle.sample_uniform(cfg.N, cfg.B, cfg.sampler_seed, t)
    assert np.array_equal(mdl.S.cpu().numpy(), S)
    rp, ci, v = oracle.induced_csr(cfg.N, rpg, cig, S)[:3]
    X_S = oracle.gather_rows(Xd.cpu().numpy(), S); y_S = oracle.gather_labels(ld.cpu().numpy(), S)
    ref = oracle.model_step(rp, ci, v, X_S, y_S, _to_np(params), drop_q=q, drop_seed=5, step=t, eps=1e-6, bf16=bf16)
    for l in range(mdl.L):
        assert rel_err(mdl.T[l].cpu().numpy(), ref["T"][l]) < tol, ("T", l)
        assert rel_err(mdl.Z[l].cpu().numpy(), ref["Z"][l]) < tol, ("Z", l)
        assert rel_err(mdl.Xh[l + 1].cpu().numpy(), ref["Xh"][l + 1]) < tol, ("Xh", l)
    assert rel_err(mdl.O.cpu().numpy(), ref["O"]) < tol
    assert abs(mdl.loss.item() - ref["loss"]) < tol * abs(ref["loss"])
    # gradients: elements whose ReLU decision differs between the two sides (pre-activation within rounding
    # distance of zero) would each move one gradient entry by a full term; the inputs are chosen so that none does
    for l in range(mdl.L):
        gam = params["layers"][l][1].double().numpy()
        got = (mdl.Z[l].cpu().numpy().astype(np.float64) * gam) > 0
        assert np.array_equal(got, (ref["Z"][l] * gam) > 0), "ReLU decisions differ: pick other inputs"
    assert rel_err(mdl.g["W_out"].cpu().numpy(), ref["dW_out"]) < tol
    assert rel_err(mdl.g["W_in"].cpu().numpy(), ref["dW_in"]) < tol
    for l in range(mdl.L):
        assert rel_err(mdl.g["layers"][l][0].cpu().numpy(), ref["dW"][l]) < tol, ("dW", l)
        assert rel_err(mdl.g["layers"][l][1].cpu().numpy(), ref["dgamma"][l]) < tol, ("dgamma", l)
    assert rel_err(mdl.dXh0.cpu().numpy(), ref["dXh0"]) < tol


def test_sgd_training_follows_the_oracle_for_a_few_steps():
    cfg, gd, Xd, ld, params = _model_inputs(seed=1)
    lr = 0.05
    mdl = sg.ScaleGnnModel(cfg.N, gd.rowptr, gd.colidx, Xd, ld, _to_dev(params), cfg.B, sampler_seed=7, drop_q=0.1,
                           drop_seed=9, optimizer="sgd", lr=lr, device=DEV)
    pn = _to_np(params)
    rpg, cig, Xh, lh = gd.rowptr.cpu().numpy(), gd.colidx.cpu().numpy(), Xd.cpu().numpy(), ld.cpu().numpy()
    for t in range(4):
        mdl.step(t)
        S = oracle.sample_uniform(cfg.N, cfg.B, 7, t)
        rp, ci, v = oracle.induced_csr(cfg.N, rpg, cig, S)[:3]
        ref = oracle.model_step(rp, ci, v, oracle.gather_rows(Xh, S), oracle.gather_labels(lh, S), pn, drop_q=0.1,
                                drop_seed=9, step=t)
        assert abs(mdl.loss.item() - ref["loss"]) < 1e-4 * abs(ref["loss"]), t
        pn = {"W_in": oracle.sgd_step(pn["W_in"], ref["dW_in"], lr), "W_out": oracle.sgd_step(pn["W_out"], ref["dW_out"], lr),
              "layers": [(oracle.sgd_step(W, ref["dW"][l], lr), oracle.sgd_step(g, ref["dgamma"][l], lr))
                         for l, (W, g) in enumerate(pn["layers"])]}
    assert rel_err(mdl.p["W_in"].cpu().numpy(), pn["W_in"]) < 1e-4
    assert rel_err(mdl.p["layers"][0][0].cpu().numpy(), pn["layers"][0][0]) < 1e-4


def test_overlapped_training_matches_step_by_step():
    # the mini-batch of step t+1 built on a second stream while step t trains: the same parameters, bit for bit,
    # after more steps than there are buffer sets, twice in a row
    cfg, gd, Xd, ld, params = _model_inputs(seed=3)
    kw = dict(sampler_seed=5, drop_q=0.1, drop_seed=3, optimizer="adam", lr=1e-3, device=DEV)
    a = sg.ScaleGnnModel(cfg.N, gd.rowptr, gd.colidx, Xd, ld, _to_dev(params), cfg.B, **kw)
    b = sg.ScaleGnnModel(cfg.N, gd.rowptr, gd.colidx, Xd, ld, _to_dev(params), cfg.B, **kw)
    for first, n in ((0, 5), (5, 4)):
        for t in range(first, first + n):
            a.step(t)
        b.run(range(first, first + n))
        torch.cuda.synchronize()
        assert torch.equal(a.loss, b.loss)
        assert torch.equal(a.p["W_in"], b.p["W_in"]) and torch.equal(a.p["W_out"], b.p["W_out"])
        for (Wa, ga), (Wb, gb) in zip(a.p["layers"], b.p["layers"]):
            assert torch.equal(Wa, Wb) and torch.equal(ga, gb)
    a.ctx.status(); b.ctx.status(); b.side_ctx.status()


def test_training_reduces_the_loss():
    # a few hundred Adam steps on a synthetic task (labels = arg max of fixed random projections of the features)
    cfg, gd, Xd, ld, params = _model_inputs(seed=2)
    mdl = sg.ScaleGnnModel(cfg.N, gd.rowptr, gd.colidx, Xd, ld, _to_dev(params), cfg.B, sampler_seed=11, drop_q=0.1,
                           drop_seed=13, optimizer="adam", lr=3e-3, device=DEV)
    losses = []
    for t in range(300):
        mdl.step(t)
        losses.append(mdl.loss.item())
    mdl.ctx.status()
    first, last = np.mean(losses[:10]), np.mean(losses[-10:])
    assert np.isfinite(losses).all()
    assert last < 0.5 * first, (first, last)


@pytest.mark.parametrize("Bn,Cn", [(1000, 47), (33, 1), (4096, 128)])
def test_binary_cross_entropy(Bn, Cn):
    O = _rand((Bn, Cn + 3), 1) * 5; Y = (np.random.default_rng(2).random((Bn, Cn)) < 0.25).astype(np.float32)
    O[0, 0] = 90.0; O[1 % Bn, 0] = -90.0          # saturated logits stay finite
    loss = torch.zeros(1, device=DEV); dO = torch.zeros((Bn, Cn), dtype=torch.float32, device=DEV)
    sg.sgnn_sigmoid_bce(ctx(), dev(O)[:, :Cn], dev(Y), loss, dO)
    lref, dref = oracle.sigmoid_bce(O[:, :Cn], Y)
    assert abs(loss.item() - lref) < TOL_F32 * abs(lref)
    assert rel_err(dO.cpu().numpy(), dref) < TOL_F32
