"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si

DEV = "cuda:0"
TOL_F32 = 1e-5     # relative error bar for fp32 features and gradients
TOL_BF16 = 2e-2    # relative error bar with bfloat16 GEMM operands
TOL_VAL = 1e-6     # edge weights (fp64 formula rounded once to fp32 on both sides)
LOGIT_BAND = 2.0 ** -7   # accuracy of a logit relative to its row's largest, bfloat16 operands and storage (checked where it is used)

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = sg.Context(0)
        # generous scratch for every test shape (vertices, stored entries, sample, width, mini-batch entries)
        _ctx.reserve(1 << 21, 1 << 25, 1 << 18, 1024, 1 << 23)
    return _ctx


def rel_err(got, ref):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    nref = np.linalg.norm(ref)
    fro = np.linalg.norm(got - ref) / (nref if nref > 0 else 1.0)
    mref = np.abs(ref).max()
    mx = np.abs(got - ref).max() / (mref if mref > 0 else 1.0)
    return max(fro, mx)


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def gpu_sample(N, B, seed, step):
    W = (N + 63) // 64
    S = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    bitmap = torch.full((W,), -1, dtype=torch.int64, device=DEV)
    rank = torch.full((W,), -1, dtype=torch.int32, device=DEV)
    ctx().reserve(N, 1, B, 1)
    sg.sgnn_sample_uniform(ctx(), N, B, seed, step, S, bitmap, rank)
    ctx().status()
    return S, bitmap, rank


def bitmap_rank_from_sample(N, S):
    """Expected bitmap words (as int64 bit patterns) and exclusive rank prefix for a sample."""
    W = (N + 63) // 64
    bits = np.zeros(W * 64, np.uint8)
    bits[np.asarray(S, np.int64)] = 1
    words = np.packbits(bits.reshape(W, 64), axis=1, bitorder="little").view(np.uint64).reshape(W)
    pop = bits.reshape(W, 64).sum(1)
    rank = np.concatenate([[0], np.cumsum(pop)[:-1]]).astype(np.int32)
    return words.view(np.int64), rank
