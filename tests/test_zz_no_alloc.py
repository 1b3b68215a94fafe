"""The allocation-free sampler entry point against the context-based one (same kernels, scratch in a
file-scope device array instead of the context's arena): two calls in a row, the second on a smaller
input, outputs bit for bit."""
import pytest
import torch

import numpy as np

import oracle
import paper_2604_02651_amd as sg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _outputs(N, B):
    W = (N + 63) // 64
    return (torch.full((B,), -1, dtype=torch.int32, device=DEV), torch.full((W,), -1, dtype=torch.int64, device=DEV),
            torch.full((W,), -1, dtype=torch.int32, device=DEV))


def _compare(ctx, N, B, seed, step):
    print("sample_uniform_static N=%d B=%d seed=%d step=%d" % (N, B, seed, step), flush=True)
    ctx.reserve(N, 1, B, 8)
    S0, bm0, rk0 = _outputs(N, B)
    sg.sgnn_sample_uniform(ctx, N, B, seed, step, S0, bm0, rk0)
    S1, bm1, rk1 = _outputs(N, B)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    sg.sgnn_sample_uniform_static(N, B, seed, step, S1, bm1, rk1, status)
    torch.cuda.synchronize()
    ctx.status()
    assert int(status.item()) == 0
    assert torch.equal(S0, S1) and torch.equal(bm0, bm1) and torch.equal(rk0, rk1)
    if N <= 100_000:
        assert np.array_equal(S1.cpu().numpy(), oracle.sample_uniform(N, B, seed, step))
    assert int(S1.min()) >= 0 and int(S1.max()) < N and bool((S1[1:] > S1[:-1]).all())


def test_static_sampler_matches_the_context_one_twice_in_a_row():
    ctx = sg.Context(0)
    try:
        _compare(ctx, 3_000_017, 200_003, 5, 11)       # several workgroups per pass, ragged last bitmap word
        _compare(ctx, 70_001, 4_099, 5, 12)            # smaller input right after: stale scratch must not show
        _compare(ctx, 65, 65, 0, 0)                    # B = N
        _compare(ctx, 1, 1, 3, 4)
        # without a status word
        S0, bm0, rk0 = _outputs(5000, 100)
        S1, bm1, rk1 = _outputs(5000, 100)
        ctx.reserve(5000, 1, 100, 8)
        sg.sgnn_sample_uniform(ctx, 5000, 100, 1, 2, S0, bm0, rk0)
        sg.sgnn_sample_uniform_static(5000, 100, 1, 2, S1, bm1, rk1)
        torch.cuda.synchronize()
        assert torch.equal(S0, S1) and torch.equal(bm0, bm1) and torch.equal(rk0, rk1)
    finally:
        ctx.close()


def test_static_sampler_rejects_what_it_cannot_hold():
    S, bm, rk = _outputs(1024, 16)
    with pytest.raises(sg.SgnnError) as e:
        sg.sgnn_sample_uniform_static((1 << 27) + 1, 16, 0, 0, S, torch.empty(((1 << 27) + 64) // 64, dtype=torch.int64, device=DEV),
                                      torch.empty(((1 << 27) + 64) // 64, dtype=torch.int32, device=DEV))
    assert e.value.code == -2 and "exceeds" in str(e.value)
    with pytest.raises(sg.SgnnError) as e:
        sg.sgnn_sample_uniform_static(1024, 0, 0, 0, S, bm, rk)
    assert e.value.code == -1
    with pytest.raises(sg.SgnnError):
        sg.sgnn_sample_uniform_static(1024, 2000, 0, 0, torch.empty(2000, dtype=torch.int32, device=DEV), bm, rk)
