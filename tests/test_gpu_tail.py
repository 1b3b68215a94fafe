"""HIP layer tail (RMSNorm + ReLU + dropout + residual, Eqs. 7-10, and its backward) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_02651_amd as sg
from gpu_util import DEV, TOL_F32, ctx
from helpers import rel_err

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def dev(a, dtype=torch.float32):
    return torch.tensor(np.ascontiguousarray(a), dtype=dtype, device=DEV)


SHAPES = [(1000, 256), (333, 100), (77, 47), (64, 2048), (4100, 128), (5, 3), (257, 32), (129, 260)]


@pytest.mark.parametrize("q", [0.0, 0.25, 0.5])
@pytest.mark.parametrize("Bn,d", SHAPES)
def test_tail_forward_backward(Bn, d, q):
    ctx().reserve(1, 1, 1024, 2048)
    Z = _rand((Bn, d), 1); g = (1.0 + 0.5 * _rand(d, 2)).astype(np.float32); R = _rand((Bn, d), 3); dY = _rand((Bn, d), 4)
    eps, seed, layer, step = 1e-6, 0xABCDEF0123, 2, 13
    Y = torch.full((Bn, d), 9.0, dtype=torch.float32, device=DEV)
    ir = torch.zeros(Bn, dtype=torch.float32, device=DEV)
    sg.sgnn_tail_fwd(ctx(), dev(Z), dev(g), eps, dev(R), q, seed, layer, step, Y, ir)
    Y_ref, ir_ref, Xn = oracle.tail_fwd(Z, gamma=g, eps=eps, R=R, q=q, seed=seed, layer=layer, step=step)
    assert rel_err(Y.cpu().numpy(), Y_ref) < TOL_F32
    assert rel_err(ir.cpu().numpy(), ir_ref) < TOL_F32
    # the dropped / clamped elements are exactly the oracle's (integer decisions; Z is the same on both sides)
    keep = oracle.dropout_keep(seed, layer, step, Bn * d, q).reshape(Bn, d) if q > 0 else np.ones((Bn, d), bool)
    zero_ref = ~(keep & (Xn > 0))
    assert np.array_equal(Y.cpu().numpy()[zero_ref], R[zero_ref])
    # backward
    dZ = torch.full((Bn, d), 9.0, dtype=torch.float32, device=DEV)
    dg = torch.zeros(d, dtype=torch.float32, device=DEV); db = torch.zeros(d, dtype=torch.float32, device=DEV)
    sg.sgnn_tail_bwd(ctx(), dev(Z), dev(ir_ref), dev(g), q, seed, layer, step, dev(dY), dZ, dg, db)
    dZ_ref, dg_ref = oracle.tail_bwd(Z, dY, gamma=g, eps=eps, q=q, seed=seed, layer=layer, step=step)
    assert rel_err(dZ.cpu().numpy(), dZ_ref) < TOL_F32
    assert rel_err(dg.cpu().numpy(), dg_ref) < TOL_F32
    assert rel_err(db.cpu().numpy(), dZ_ref.sum(axis=0)) < TOL_F32
    # bit-reproducible, and the sums are optional
    dZ2 = torch.zeros_like(dZ); dg2 = torch.zeros_like(dg)
    sg.sgnn_tail_bwd(ctx(), dev(Z), dev(ir_ref), dev(g), q, seed, layer, step, dev(dY), dZ2, dg2, None)
    assert torch.equal(dZ, dZ2) and torch.equal(dg, dg2)
    sg.sgnn_tail_bwd(ctx(), dev(Z), dev(ir_ref), dev(g), q, seed, layer, step, dev(dY), dZ2, None, None)
    assert torch.equal(dZ, dZ2)


def test_tail_without_scale_residual_and_with_strides():
    Bn, d = 300, 96
    Z = _rand((Bn, d + 4), 5); dY = _rand((Bn, d), 6)
    Zd = dev(Z)[:, :d]
    Yfull = torch.full((Bn, d + 8), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_tail_fwd(ctx(), Zd, None, 0.0, None, 0.0, 0, 0, 0, Yfull[:, :d], None)
    Y_ref, ir_ref, _ = oracle.tail_fwd(Z[:, :d], eps=0.0)
    assert rel_err(Yfull[:, :d].cpu().numpy(), Y_ref) < TOL_F32
    assert torch.all(Yfull[:, d:] == 9.0)
    dZ = torch.zeros((Bn, d), dtype=torch.float32, device=DEV)
    sg.sgnn_tail_bwd(ctx(), Zd, dev(ir_ref), None, 0.0, 0, 0, 0, dev(dY), dZ, None, None)
    assert rel_err(dZ.cpu().numpy(), oracle.tail_bwd(Z[:, :d], dY, eps=0.0)[0]) < TOL_F32


def test_tail_rejects_bad_arguments():
    Z = dev(_rand((8, 16), 1)); Y = torch.zeros_like(Z)
    with pytest.raises(sg.SgnnError):
        sg.sgnn_tail_fwd(ctx(), Z, None, 1e-6, None, 1.0, 0, 0, 0, Y, None)          # drop probability 1
    with pytest.raises(sg.SgnnError):
        sg.sgnn_tail_fwd(ctx(), Z, None, 1e-6, None, 0.1, 0, 0, 0, torch.zeros((8, 17), device=DEV), None)
    wide = dev(_rand((2, 2052), 2))
    with pytest.raises(sg.SgnnError):
        sg.sgnn_tail_fwd(ctx(), wide, None, 1e-6, None, 0.0, 0, 0, 0, torch.zeros_like(wide), None)


@pytest.mark.parametrize("fuse", [True, False])
@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("q", [0.0, 0.3])
@pytest.mark.parametrize("M,K,N", [(5000, 256, 256), (4100, 100, 128), (4096, 64, 64), (9001, 172, 200), (700, 64, 64),
                                   (4500, 256, 47)])
def test_transform_and_tail_in_one_call(M, K, N, q, bf16, fuse):
    # with SGNN_FUSE_TAIL tall bf16 products run the tail in the epilogue of the product (one kernel); the other
    # shapes, fp32 and the default run the two kernels one after the other.  Either way: Z = T W, Y = tail(Z).
    ctx().reserve(1, 1, 16384, 256)
    T = _rand((M, K), 1); W = (_rand((K, N), 2) / np.sqrt(K)).astype(np.float32)
    g = (1.0 + 0.5 * _rand(N, 3)).astype(np.float32); R = _rand((M, N), 4)
    seed, layer, step, eps = 12345, 1, 7, 1e-6
    Z = torch.zeros((M, N), dtype=torch.float32, device=DEV); Y = torch.zeros_like(Z)
    ir = torch.zeros(M, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm_tail_fwd(ctx(), dev(T), dev(W), dev(g), eps, dev(R), q, seed, layer, step,
                          (sg.SGNN_BF16_MFMA if bf16 else 0) | (sg.SGNN_FUSE_TAIL if fuse else 0), Z, Y, ir)
    rd = oracle.round_bf16 if bf16 else (lambda x: x.astype(np.float64))
    Z_ref = oracle.gemm(rd(T), rd(W))
    assert rel_err(Z.cpu().numpy(), Z_ref) < (1e-4 if bf16 else TOL_F32)
    # the tail of the Z the kernels produced (so that the ReLU and dropout decisions are those of the same values)
    Zk = Z.cpu().numpy()
    Y_ref, ir_ref, _ = oracle.tail_fwd(Zk, gamma=g, eps=eps, R=R, q=q, seed=seed, layer=layer, step=step)
    assert rel_err(Y.cpu().numpy(), Y_ref) < TOL_F32
    assert rel_err(ir.cpu().numpy(), ir_ref) < TOL_F32
