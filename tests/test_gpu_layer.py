"""GPU parity: SpMM, MFMA GEMM, layer forward / backward and the whole step against the CPU oracle."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
import paper_2604_02651_amd as sg
import synth_inputs as si
from gpu_util import DEV, LOGIT_BAND, TOL_BF16, TOL_F32, TOL_VAL, ctx, dev, rel_err

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _sub_csr(N=3000, edges=40000, B=1500, seed=5):
    g = si.rmat_graph(N, edges, seed=seed)
    S = oracle.sample_uniform(N, B, 0, 0)
    rp, ci, v = oracle.induced_csr(N, g.rowptr.numpy(), g.colidx.numpy(), S)
    return B, rp, ci, v


@pytest.fixture(scope="module")
def sub():
    return _sub_csr()


@pytest.mark.parametrize("d", [1, 3, 8, 32, 41, 47, 64, 100, 128, 172, 256, 602, 1024])
def test_spmm_widths(sub, d):
    B, rp, ci, v = sub
    ctx().reserve(B, len(ci), B, d, len(ci))
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    X = _rand((B, d), d)
    out = torch.full((B, d), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, dev(X), out)
    ref = oracle.spmm(rp, ci, v, X.astype(np.float64))
    assert rel_err(out.cpu().numpy(), ref) < TOL_F32


@pytest.mark.parametrize("d", [3, 32, 47, 100, 128, 256, 602])
def test_spmm_bfloat16_input(sub, d):
    # the input operand stored as bfloat16 (features of the largest configuration), read through a row index
    B, rp, ci, v = sub
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    ctx().reserve(B, len(ci), B, d, len(ci))
    big = dev(_rand((4000, d), 2 + d)).to(torch.bfloat16)
    idx = np.random.default_rng(3).permutation(4000)[:B].astype(np.int32)
    out = torch.full((B, d), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, big, out, row_index=dev(idx))
    ref = oracle.spmm(rp, ci, v, big.float().cpu().numpy()[idx].astype(np.float64))
    assert rel_err(out.cpu().numpy(), ref) < TOL_F32        # the stored values are the inputs: only the fp32 sum differs
    plain = big[torch.as_tensor(idx.astype(np.int64), device=DEV)].contiguous()
    out2 = torch.zeros_like(out)
    sg.sgnn_spmm(ctx(), A, plain, out2)
    assert torch.equal(out, out2)


def test_spmm_row_index_and_padding(sub):
    B, rp, ci, v = sub
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    big = _rand((5000, 130), 1)           # leading dimension 130, logical width 128
    idx = np.random.default_rng(2).permutation(5000)[:B].astype(np.int32)
    Xd = dev(big)[:, :128]
    out_full = torch.zeros((B, 132), dtype=torch.float32, device=DEV)
    out = out_full[:, :128]
    sg.sgnn_spmm(ctx(), A, Xd, out, row_index=dev(idx))
    ref = oracle.spmm(rp, ci, v, big[idx][:, :128].astype(np.float64))
    assert rel_err(out.cpu().numpy(), ref) < TOL_F32
    assert torch.all(out_full[:, 128:] == 0)


def test_spmm_rectangular_empty_rows_and_long_row():
    rows, cols, d = 70, 5000, 64
    rng = np.random.default_rng(0)
    lists = [np.zeros(0, np.int32) for _ in range(rows)]
    lists[3] = np.sort(rng.permutation(cols)[:4500]).astype(np.int32)      # one very long row
    for i in range(10, 70, 3):
        lists[i] = np.sort(rng.permutation(cols)[:rng.integers(1, 9)]).astype(np.int32)
    rp = np.concatenate([[0], np.cumsum([len(x) for x in lists])]).astype(np.int32)
    ci = np.concatenate(lists); v = rng.standard_normal(len(ci)).astype(np.float32)
    A = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV)
    X = _rand((cols, d), 3)
    out = torch.full((rows, d), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, dev(X), out)
    assert rel_err(out.cpu().numpy(), oracle.spmm(rp, ci, v, X.astype(np.float64))) < TOL_F32


@pytest.mark.parametrize("d", [32, 100, 256, 602])
def test_spmm_rows_of_every_length_class(d):
    # rows walked by one lane group, rows shared by a workgroup, rows cut into chunks (one of them
    # starting exactly on a chunk boundary), empty rows in between
    rng = np.random.default_rng(7)
    rows, cols = 300, 9000
    lens = rng.integers(0, 5, rows)
    lens[[5, 17, 40]] = [65, 300, 512]
    lens[[60, 61, 90, 299]] = [513, 2000, 5000, 1300]
    lens[0] = 1024 - 0
    lists = [np.sort(rng.permutation(cols)[:n]).astype(np.int32) for n in lens]
    rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci = np.concatenate(lists); v = rng.standard_normal(len(ci)).astype(np.float32)
    A = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV)
    X = _rand((cols, d), 3)
    out = torch.full((rows, d), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, dev(X), out)
    assert rel_err(out.cpu().numpy(), oracle.spmm(rp, ci, v, X.astype(np.float64))) < TOL_F32
    out2 = torch.zeros_like(out)
    sg.sgnn_spmm(ctx(), A, dev(X), out2)
    assert torch.equal(out, out2)          # bit-reproducible
    # with a plan attached to the matrix (built once) the result is the same
    Ap = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV, with_plan=True)
    sg.sgnn_csr_plan(ctx(), Ap)
    out3 = torch.zeros_like(out)
    sg.sgnn_spmm(ctx(), Ap, dev(X), out3)
    sg.sgnn_spmm(ctx(), Ap, dev(X), out3)
    assert torch.equal(out, out3)


@pytest.mark.parametrize("d", [47, 256])
def test_spmm_hub_rows_get_longer_pieces(d):
    # rows beyond 256 pieces of 64 entries are cut into longer pieces: one row right at the limit, one
    # just beyond it, one far beyond it
    rng = np.random.default_rng(13)
    rows, cols = 40, 70000
    lens = rng.integers(0, 4, rows)
    lens[[3, 10, 11, 39]] = [50000, 16385, 16384, 33000]
    lists = [np.sort(rng.choice(cols, n, replace=False)).astype(np.int32) for n in lens]
    rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci = np.concatenate(lists); v = rng.standard_normal(len(ci)).astype(np.float32)
    ctx().reserve(cols, len(ci), rows, d, len(ci))
    A = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV, with_plan=True)
    sg.sgnn_csr_plan(ctx(), A)
    X = _rand((cols, d), 3)
    out = torch.full((rows, d), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, dev(X), out)
    assert rel_err(out.cpu().numpy(), oracle.spmm(rp, ci, v, X.astype(np.float64))) < TOL_F32
    out2 = torch.zeros_like(out)
    sg.sgnn_spmm(ctx(), A, dev(X), out2)
    assert torch.equal(out, out2)


@pytest.mark.parametrize("d", [32, 256])
def test_spmm_many_long_rows_repeated(d):
    # thousands of pieces of long rows in flight on all compute dies, their partial rows handed from
    # wavefront to wavefront inside the kernel; the tickets of the plan are used again by every product
    rng = np.random.default_rng(11)
    rows, cols = 3000, 20000
    lens = rng.integers(0, 6, rows)
    long_rows = rng.permutation(rows)[:700]
    lens[long_rows] = rng.integers(65, 1500, len(long_rows))
    lists = [np.sort(rng.choice(cols, n, replace=False)).astype(np.int32) for n in lens]
    rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci = np.concatenate(lists); v = rng.standard_normal(len(ci)).astype(np.float32)
    ctx().reserve(cols, len(ci), rows, d, len(ci))
    A = sg.Csr.from_arrays(rows, cols, rp, ci, v, DEV, with_plan=True)
    sg.sgnn_csr_plan(ctx(), A)
    X = dev(_rand((cols, d), 3))
    first = torch.zeros((rows, d), dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(ctx(), A, X, first)
    assert rel_err(first.cpu().numpy(), oracle.spmm(rp, ci, v, X.cpu().numpy().astype(np.float64))) < TOL_F32
    out = torch.empty_like(first)
    for _ in range(40):
        out.fill_(-1.0)
        sg.sgnn_spmm(ctx(), A, X, out)
        assert torch.equal(out, first)


def test_scratch_too_small_is_an_error():
    small = sg.Context(0)
    B, rp, ci, v = _sub_csr(500, 3000, 200, 1)
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    A.capacity = 100000        # pretend a large entry array: the chunk scratch no longer fits
    A.colidx = torch.zeros(100000, dtype=torch.int32, device=DEV); A.val = torch.zeros(100000, dtype=torch.float32, device=DEV)
    with pytest.raises(sg.SgnnError) as e:
        sg.sgnn_spmm(small, A, dev(_rand((B, 8), 1)), torch.zeros((B, 8), dtype=torch.float32, device=DEV))
    assert e.value.code == -2
    small.close()


GEMM_SHAPES = [(1, 1, 1), (5, 7, 3), (33, 65, 17), (128, 128, 16), (130, 129, 100), (257, 32, 256), (300, 8, 64),
               (1000, 47, 256), (513, 256, 602), (2048, 172, 128), (64, 41, 33)]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_nn_with_epilogue(M, N, K, bf16):
    A = _rand((M, K), 1); Bm = _rand((K, N), 2); bias = _rand(N, 3)
    C = torch.full((M, N), 9.0, dtype=torch.float32, device=DEV)
    flags = sg.SGNN_RELU | (sg.SGNN_BF16_MFMA if bf16 else 0)
    sg.sgnn_gemm(ctx(), False, False, dev(A), dev(Bm), dev(bias), flags, C)
    A64, B64 = A.astype(np.float64), Bm.astype(np.float64)
    if bf16:
        A64, B64 = oracle.round_bf16(A), oracle.round_bf16(Bm)
    ref = np.maximum(oracle.gemm(A64, B64) + bias, 0)
    # with identically rounded operands only the fp32 accumulation differs
    assert rel_err(C.cpu().numpy(), ref) < (TOL_F32 if not bf16 else 1e-4)
    if bf16:
        full = np.maximum(A.astype(np.float64) @ Bm.astype(np.float64) + bias, 0)
        assert rel_err(C.cpu().numpy(), full) < TOL_BF16


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_nt_and_tn(M, N, K, bf16):
    flags = sg.SGNN_BF16_MFMA if bf16 else 0
    rd = oracle.round_bf16 if bf16 else (lambda x: x.astype(np.float64))
    tol = 1e-4 if bf16 else TOL_F32
    A = _rand((M, K), 4); Bt = _rand((N, K), 5)
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, flags, C)
    assert rel_err(C.cpu().numpy(), rd(A) @ rd(Bt).T) < tol
    At = _rand((K, M), 6); Bm = _rand((K, N), 7)
    C2 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, flags, C2)
    assert rel_err(C2.cpu().numpy(), rd(At).T @ rd(Bm)) < tol


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,N,K", [(1000, 256, 32), (300, 172, 128), (5000, 256, 256), (77, 40, 8), (4100, 100, 47)])
def test_gemm_masked_result(M, N, K, bf16):
    # the ReLU backward of the layer below applied while the input gradient dP W^T is written
    flags = sg.SGNN_BF16_MFMA if bf16 else 0
    rd = oracle.round_bf16 if bf16 else (lambda x: x.astype(np.float64))
    A = _rand((M, K), 14); Bt = _rand((N, K), 15)
    mask = np.maximum(_rand((M, N + 3), 16), 0.0)          # about half the entries are zero, as after a ReLU
    C = torch.full((M, N), 5.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, flags, C, mask=dev(mask)[:, :N])
    ref = np.where(mask[:, :N] > 0, rd(A) @ rd(Bt).T, 0.0)
    assert rel_err(C.cpu().numpy(), ref) < (1e-4 if bf16 else TOL_F32)
    assert torch.all(C[dev(mask)[:, :N] <= 0] == 0)


@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("M,N,K", [(5000, 256, 172), (4096, 256, 256), (9001, 172, 256), (4100, 100, 47), (6000, 36, 128),
                                   (4500, 64, 200)])
def test_gemm_tall_bf16_masked_in_chunks(M, N, K, tb):
    # the tall-operand bf16 kernel with a mask it can read 16 bytes at a time (aligned, leading dimension a multiple of
    # four): every column-tile and slice count of the kernel, a ragged last row block, a mask wider than the result
    A = _rand((M, K), 21); Bm = _rand((N, K) if tb else (K, N), 22)
    mask = np.maximum(_rand((M, N + 4), 23), 0.0)
    md = dev(mask)[:, :N]
    assert md.stride(0) % 4 == 0 and md.data_ptr() % 16 == 0
    C = torch.full((M, N), 5.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, tb, dev(A), dev(Bm), None, sg.SGNN_BF16_MFMA, C, mask=md)
    prod = oracle.round_bf16(A) @ (oracle.round_bf16(Bm).T if tb else oracle.round_bf16(Bm))
    ref = np.where(mask[:, :N] > 0, prod, 0.0)
    assert rel_err(C.cpu().numpy(), ref) < 1e-4
    assert torch.all(C[md <= 0] == 0)


def _bf(x):
    return torch.as_tensor(np.ascontiguousarray(x)).to(torch.bfloat16)


@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("M,N,K", [(5000, 256, 172), (4096, 256, 256), (9001, 172, 256), (4100, 100, 48), (6000, 36, 128),
                                   (4500, 64, 200), (1000, 256, 128), (300, 47, 100)])
def test_gemm_bf16_stored_operand_and_result(M, N, K, tb):
    # A and C stored as bfloat16 (tall shapes: the kernel reads and writes them; short ones: fp32 copies in scratch):
    # the product of the stored values, rounded once to bfloat16 when written
    A = oracle.round_bf16(_rand((M, K), 31)); Bm = _rand((N, K) if tb else (K, N), 32); bias = _rand((N,), 33)
    Ad = _bf(np.pad(A, ((0, 0), (0, (-K) % 8)))).to(DEV)[:, :K]
    C = torch.full((M, (N + 7) // 8 * 8), 5.0, dtype=torch.bfloat16, device=DEV)[:, :N]
    ctx().reserve(1, 1, M, 256)
    sg.sgnn_gemm(ctx(), False, tb, Ad, dev(Bm), dev(bias), sg.SGNN_BF16_MFMA | sg.SGNN_RELU, C)
    Br = oracle.round_bf16(Bm)
    ref = np.maximum(A @ (Br.T if tb else Br) + bias, 0.0)
    got = C.float().cpu().numpy().astype(np.float64)
    # the kernel accumulates in fp32 and rounds once: within one bfloat16 unit of the rounded exact result
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * np.abs(ref).max())
    assert rel_err(got, oracle.round_bf16(ref)) < 2.0 ** -8
    # fp32 result from the same stored operand: to fp32 accuracy
    C32 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, tb, Ad, dev(Bm), dev(bias), sg.SGNN_BF16_MFMA | sg.SGNN_RELU, C32)
    assert rel_err(C32.cpu().numpy(), ref) < 1e-4


@pytest.mark.parametrize("M,N,K", [(5000, 256, 172), (4100, 100, 48), (700, 64, 40)])
def test_gemm_bf16_stored_mask_and_weight_gradient(M, N, K):
    # the mask stored as bfloat16 (chunked and element-wise paths), and A^T B with a bfloat16-stored A
    A = _rand((M, K), 41); Bt = _rand((N, K), 42)
    mask = oracle.round_bf16(np.maximum(_rand((M, N), 43), 0.0))
    md = _bf(np.pad(mask, ((0, 0), (0, (-N) % 8)))).to(DEV)[:, :N]
    C = torch.full((M, N), 5.0, dtype=torch.float32, device=DEV)
    ctx().reserve(1, 1, M, 256)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, sg.SGNN_BF16_MFMA, C, mask=md)
    ref = np.where(mask > 0, oracle.round_bf16(A) @ oracle.round_bf16(Bt).T, 0.0)
    assert rel_err(C.cpu().numpy(), ref) < 1e-4 and torch.all(C[md <= 0] == 0)
    # dW = T^T dZ with T stored as bfloat16 (M rows reduced), with the column sums of dZ
    T = oracle.round_bf16(_rand((M, K), 44)); dZ = _rand((M, N), 45)
    Td = _bf(np.pad(T, ((0, 0), (0, (-K) % 8)))).to(DEV)[:, :K]
    dW = torch.zeros((K, N), dtype=torch.float32, device=DEV); cs = torch.zeros(N, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, Td, dev(dZ), None, sg.SGNN_BF16_MFMA, dW, b_colsum=cs)
    assert rel_err(dW.cpu().numpy(), T.T @ oracle.round_bf16(dZ)) < 1e-4
    assert rel_err(cs.cpu().numpy(), dZ.astype(np.float64).sum(axis=0)) < 1e-4
    dW32 = torch.zeros_like(dW)
    sg.sgnn_gemm(ctx(), True, False, dev(T, torch.float32), dev(dZ), None, sg.SGNN_BF16_MFMA, dW32)
    assert torch.equal(dW, dW32)          # the stored values are what the fp32-stored operand rounds to: same product
    # B stored as bfloat16 as well (the gradient handed down by the layer above); its column sums are those of the stored values
    dZr = oracle.round_bf16(dZ)
    dZd = _bf(np.pad(dZr, ((0, 0), (0, (-N) % 8)))).to(DEV)[:, :N]
    for Aop in (Td, dev(T, torch.float32)):
        dWb = torch.zeros_like(dW); csb = torch.zeros_like(cs)
        sg.sgnn_gemm(ctx(), True, False, Aop, dZd, None, sg.SGNN_BF16_MFMA, dWb, b_colsum=csb)
        assert torch.equal(dWb, dW)
        assert rel_err(csb.cpu().numpy(), dZr.sum(axis=0)) < 1e-5
    # the masked input gradient written as bfloat16 from a bfloat16-stored operand
    Ab = oracle.round_bf16(A)
    Abd = _bf(np.pad(Ab, ((0, 0), (0, (-K) % 8)))).to(DEV)[:, :K]
    C16 = torch.full((M, (N + 7) // 8 * 8), 5.0, dtype=torch.bfloat16, device=DEV)[:, :N]
    sg.sgnn_gemm(ctx(), False, True, Abd, dev(Bt), None, sg.SGNN_BF16_MFMA, C16, mask=md)
    got = C16.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * np.abs(ref).max()) and torch.all(C16[md <= 0] == 0)


@pytest.mark.parametrize("K,M,N", [(16384, 256, 256), (40000 // 32 * 32, 128, 256), (8192, 256, 172), (12000 // 32 * 32, 100, 48),
                                   (65536, 4, 2), (9984, 130, 66), (8192, 256, 8), (32768, 36, 250),
                                   (16384, 256, 47), (8192, 255, 3), (8192, 64, 255)])   # odd widths: one store per value
def test_weight_gradient_of_bf16_stored_operands_streams(K, M, N):
    # A^T B with both operands stored as bfloat16 and a long reduction: the streaming kernel (every frame size up to
    # 256 x 256, leading dimensions with and without padding, wavefronts with nothing to do), with the column sums of B;
    # fixed split and summation order: bit-reproducible
    A = oracle.round_bf16(_rand((K, M), 61)); Bm = oracle.round_bf16(_rand((K, N), 62))
    Ad = _bf(np.pad(A, ((0, 0), (0, (-M) % 8)))).to(DEV)[:, :M]
    Bd = _bf(np.pad(Bm, ((0, 0), (0, (-N) % 8)))).to(DEV)[:, :N]
    ctx().reserve(1, 1, K, 256)
    C = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV); cs = torch.full((N,), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, Ad, Bd, None, sg.SGNN_BF16_MFMA, C, b_colsum=cs)
    assert rel_err(C.cpu().numpy(), A.T @ Bm) < 1e-5
    assert np.abs(cs.cpu().numpy() - Bm.sum(axis=0)).max() < 1e-5 * np.abs(Bm).sum(axis=0).max()
    C2 = torch.zeros_like(C); cs2 = torch.zeros_like(cs)
    sg.sgnn_gemm(ctx(), True, False, Ad, Bd, None, sg.SGNN_BF16_MFMA, C2, b_colsum=cs2)
    assert torch.equal(C, C2) and torch.equal(cs, cs2)
    C3 = torch.zeros_like(C)
    sg.sgnn_gemm(ctx(), True, False, Ad, Bd, None, sg.SGNN_BF16_MFMA, C3)          # without the column sums
    assert torch.equal(C, C3)
    # the same product from fp32-stored copies of the same values (the tile kernel): equal up to summation order
    C4 = torch.zeros_like(C)
    sg.sgnn_gemm(ctx(), True, False, dev(A, torch.float32), dev(Bm, torch.float32), None, sg.SGNN_BF16_MFMA, C4)
    assert rel_err(C4.cpu().numpy(), C.cpu().numpy().astype(np.float64)) < 1e-5


@pytest.mark.parametrize("d", [256, 172, 128, 100, 47, 33])
def test_spmm_bf16_stored_result(d):
    # out stored as bfloat16: the fp32 sum rounded once; with a bfloat16 input as well
    rng = np.random.default_rng(d)
    rows = 3000
    dense = (rng.random((rows, rows)) < 0.002) * rng.random((rows, rows))
    dense[5, :] = rng.random(rows) * (rng.random(rows) < 0.5)           # a long row: pieces and the last-ticket sum
    A = sp.csr_matrix(dense.astype(np.float32))
    X = oracle.round_bf16(_rand((rows, d), 51))
    Ad = sg.Csr.from_arrays(rows, rows, A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float32), DEV)
    ctx().reserve(rows, A.nnz, rows, max(d, 8), A.nnz)
    want = oracle.spmm(A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float32), X)
    for xin in (dev(X, torch.float32), _bf(np.pad(X, ((0, 0), (0, (-d) % 8)))).to(DEV)[:, :d]):
        out = torch.full((rows, (d + 7) // 8 * 8), 3.0, dtype=torch.bfloat16, device=DEV)[:, :d]
        sg.sgnn_spmm(ctx(), Ad, xin, out)
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(want).max())


@pytest.mark.parametrize("d", [8, 41, 47, 64, 100, 172, 256, 300, 512, 173, 600])
def test_spmm_with_the_loss_in_its_epilogue(d):
    # O = A X + b, the mean cross-entropy of O and its gradient in one call: against the oracle, and against the
    # product followed by the loss kernel (per row the same arithmetic: logits and gradient rows bit for bit; the sums
    # over the rows are taken in another order).  One vector width and chunk count per column count; 173 and 600 are
    # shapes the fused kernels do not take (two kernels behind the same call); a long row goes through the pieces
    rng = np.random.default_rng(d)
    rows = 3000
    dense = (rng.random((rows, rows)) < 0.002) * rng.random((rows, rows))
    dense[5, :] = rng.random(rows) * (rng.random(rows) < 0.5)
    dense[77, :] = 0.0                                               # an empty row: logits = bias
    A = sp.csr_matrix(dense.astype(np.float32))
    rp, ci, va = A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float32)
    X = oracle.round_bf16(_rand((rows, d), 52)) * 4.0
    bias = _rand((d,), 53)
    y = rng.integers(0, d, rows).astype(np.int32)
    Ad = sg.Csr.from_arrays(rows, rows, rp, ci, va, DEV)
    ctx().reserve(rows, A.nnz, rows, max(d, 8), A.nnz)
    O_ref = oracle.spmm(rp, ci, va, X) + bias[None, :]
    l_ref, dO_ref = oracle.softmax_xent(O_ref, y)
    pad = (-d) % 8
    bd, yd = dev(bias, torch.float32), dev(y)
    for xin in (dev(np.pad(X, ((0, 0), (0, pad))), torch.float32)[:, :d], _bf(np.pad(X, ((0, 0), (0, pad)))).to(DEV)[:, :d]):
        # the two kernels one after the other
        O2 = torch.zeros((rows, d + pad), dtype=torch.float32, device=DEV)[:, :d]
        sg.sgnn_spmm(ctx(), Ad, xin, O2)
        O2 += bd
        loss2 = torch.zeros(1, dtype=torch.float32, device=DEV); dO2 = torch.zeros_like(O2); cs2 = torch.zeros(d, dtype=torch.float32, device=DEV)
        sg.sgnn_softmax_xent(ctx(), O2, yd, loss2, dO2, dO_colsum=cs2)
        # one call
        O = torch.full((rows, d + pad), 7.0, dtype=torch.float32, device=DEV)[:, :d]
        dO = torch.full((rows, d + pad), 7.0, dtype=torch.float32, device=DEV)[:, :d]
        loss = torch.zeros(1, dtype=torch.float32, device=DEV); cs = torch.zeros(d, dtype=torch.float32, device=DEV)
        sg.sgnn_spmm_xent(ctx(), Ad, xin, bd, yd, loss, dO, O=O, dO_colsum=cs)
        assert rel_err(O.cpu().numpy(), O_ref) < TOL_F32 and rel_err(dO.cpu().numpy(), dO_ref) < TOL_F32
        assert abs(loss.item() - l_ref) < TOL_F32 * abs(l_ref)
        assert np.abs(cs.cpu().numpy() - dO_ref.sum(axis=0)).max() < TOL_F32 * np.abs(dO_ref).sum(axis=0).max()
        assert rel_err(O.cpu().numpy(), O2.cpu().numpy().astype(np.float64)) < 1e-6
        assert rel_err(dO.cpu().numpy(), dO2.cpu().numpy().astype(np.float64)) < 1e-6
        # again: bit-reproducible; without the logits; gradient stored as bfloat16 (column sums of what is stored)
        dO3 = torch.zeros_like(dO); loss3 = torch.zeros_like(loss); cs3 = torch.zeros_like(cs)
        sg.sgnn_spmm_xent(ctx(), Ad, xin, bd, yd, loss3, dO3, O=None, dO_colsum=cs3)
        assert torch.equal(dO, dO3) and torch.equal(loss, loss3) and torch.equal(cs, cs3)
        dO16 = torch.zeros((rows, (d + 31) // 32 * 32), dtype=torch.bfloat16, device=DEV)[:, :d]; cs16 = torch.zeros_like(cs)
        sg.sgnn_spmm_xent(ctx(), Ad, xin, bd, yd, loss3, dO16, O=None, dO_colsum=cs16)
        assert torch.equal(dO16, dO.to(torch.bfloat16)) and torch.equal(loss, loss3)
        stored = dO16.float().cpu().numpy().astype(np.float64)
        assert np.abs(cs16.cpu().numpy() - stored.sum(axis=0)).max() < TOL_F32 * np.abs(stored).sum(axis=0).max()
        sg.sgnn_spmm_xent(ctx(), Ad, xin, None, yd, loss3, None)                       # the loss alone, no bias
        l_nb, _ = oracle.softmax_xent(O_ref - bias[None, :], y)
        assert abs(loss3.item() - l_nb) < TOL_F32 * abs(l_nb)


def test_spmm_with_the_loss_rejects_what_it_cannot_take():
    rows, d = 64, 8
    A = sp.identity(rows, dtype=np.float32, format="csr")
    Ad = sg.Csr.from_arrays(rows, rows, A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float32), DEV)
    ctx().reserve(rows, rows, rows, 8, rows)
    X = dev(_rand((rows, d), 1), torch.float32); y = dev(np.zeros(rows, np.int32))
    loss = torch.zeros(1, dtype=torch.float32, device=DEV); dO = torch.zeros((rows, d), dtype=torch.float32, device=DEV)
    with pytest.raises(ValueError):
        sg.sgnn_spmm_xent(ctx(), Ad, X, None, y[:10], loss, dO)                       # a label per row
    with pytest.raises(ValueError):
        sg.sgnn_spmm_xent(ctx(), Ad, X, None, y, loss, dO[:, :4])                     # gradient of another shape
    with pytest.raises(sg.SgnnError):
        sg.sgnn_spmm_xent(ctx(), Ad, X[:32], None, y, loss, None)                     # X must have a row per column of A
    with pytest.raises(sg.SgnnError):
        sg.sgnn_spmm_xent(ctx(), Ad, X, None, y, loss, None, dO_colsum=torch.zeros(d, device=DEV))   # column sums of no gradient
    sg.sgnn_spmm_xent(ctx(), Ad, X, None, y, loss, dO)                                # and the plain call still works
    l_ref, dO_ref = oracle.softmax_xent(X.cpu().numpy().astype(np.float64), np.zeros(rows, np.int32))
    assert abs(loss.item() - l_ref) < TOL_F32 * abs(l_ref) and rel_err(dO.cpu().numpy(), dO_ref) < TOL_F32


@pytest.mark.parametrize("bf16", [False, True])
def test_gemm_long_reduction_is_split_and_reproducible(bf16):
    # the weight-gradient shape: short result, reduction over tens of thousands of rows
    K, M, N = 40000, 100, 256
    ctx().reserve(1, 1, 40000, 256)
    At = _rand((K, M), 8); Bm = _rand((K, N), 9)
    flags = sg.SGNN_BF16_MFMA if bf16 else 0
    rd = oracle.round_bf16 if bf16 else (lambda x: x.astype(np.float64))
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, flags, C)
    assert rel_err(C.cpu().numpy(), rd(At).T @ rd(Bm)) < (1e-4 if bf16 else TOL_F32)
    C2 = torch.zeros_like(C)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, flags, C2)
    assert torch.equal(C, C2)


@pytest.mark.parametrize("M,N,K", [(1000, 256, 256), (4096, 128, 64), (300, 172, 128), (129, 68, 32), (2500, 256, 96),
                                   (777, 100, 160)])
def test_gemm_fp32_wide_results(M, N, K):
    # wide fp32 results with a reduction length that is a multiple of 32 (the direct global -> LDS tile kernel),
    # ragged in M and N, all three operand orders
    ctx().reserve(1, 1, 40000, 256)
    A = _rand((M, K), 21); Bm = _rand((K, N), 22); bias = _rand(N, 23)
    C = torch.full((M, N), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, False, dev(A), dev(Bm), dev(bias), sg.SGNN_RELU, C)
    assert rel_err(C.cpu().numpy(), np.maximum(oracle.gemm(A, Bm) + bias, 0)) < TOL_F32
    Bt = _rand((N, K), 24)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, 0, C)
    assert rel_err(C.cpu().numpy(), oracle.gemm(A, Bt.T.copy())) < TOL_F32
    At = _rand((K, M), 25)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, 0, C)
    assert rel_err(C.cpu().numpy(), oracle.gemm(At.T.copy(), Bm)) < TOL_F32


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,N,K", [(256, 256, 32768), (128, 256, 5000), (100, 64, 300), (64, 32, 40000), (33, 47, 129)])
def test_gemm_weight_gradient_with_column_sums(M, N, K, bf16):
    # dW = T^T dZ with db = column sums of dZ from the same pass (split and unsplit, chunked and masked kernels)
    ctx().reserve(1, 1, 40000, 256)
    At = _rand((K, M), 28); Bm = _rand((K, N), 29)
    flags = sg.SGNN_BF16_MFMA if bf16 else 0
    rd = oracle.round_bf16 if bf16 else (lambda x: x.astype(np.float64))
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV); cs = torch.full((N,), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, flags, C, b_colsum=cs)
    assert rel_err(C.cpu().numpy(), oracle.gemm(rd(At).T.copy(), rd(Bm))) < (1e-4 if bf16 else TOL_F32)
    assert rel_err(cs.cpu().numpy(), Bm.astype(np.float64).sum(axis=0)) < TOL_F32      # the sums are of the fp32 values
    C2 = torch.zeros_like(C); cs2 = torch.zeros_like(cs)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, flags, C2, b_colsum=cs2)
    assert torch.equal(C, C2) and torch.equal(cs, cs2)
    with pytest.raises(sg.SgnnError):
        sg.sgnn_gemm(ctx(), False, False, dev(At.T.copy()), dev(Bm), None, flags, C2, b_colsum=cs2)


@pytest.mark.parametrize("M,N,K", [(256, 32, 32768), (100, 7, 4129), (132, 32, 5000), (260, 20, 70001), (4, 1, 4096),
                                   (128, 32, 9000), (256, 64, 8192), (132, 100, 5001), (512, 256, 4096), (260, 34, 4500),
                                   (128, 256, 32768)])
def test_gemm_fp32_narrow_weight_gradient(M, N, K):
    # A^T B with a small result (a few tiles of 128 x 32 or 128 x 64) and a long reduction: operands go from memory
    # straight into the matrix-core layout; ragged in every dimension, with and without the column sums of B
    ctx().reserve(1, 1, 70001, 272)
    pad = 1 if N <= 32 else 4          # wider results need 16-byte aligned rows of B, narrow ones take any
    At = _rand((K, M + 4), 41)[:, :M]; Bm = _rand((K, N + pad), 42)[:, :N]
    C = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV); cs = torch.full((N,), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, dev(_rand((K, M + 4), 41))[:, :M], dev(_rand((K, N + pad), 42))[:, :N], None, 0, C, b_colsum=cs)
    ref = oracle.gemm(At.T.copy(), Bm.copy())
    assert rel_err(C.cpu().numpy(), ref) < TOL_F32
    # a sum of thousands of signed terms cancels: the error is measured against the sum of their magnitudes
    B64 = Bm.astype(np.float64)
    assert np.abs(cs.cpu().numpy() - B64.sum(axis=0)).max() < TOL_F32 * np.abs(B64).sum(axis=0).max()
    C2 = torch.zeros_like(C)
    sg.sgnn_gemm(ctx(), True, False, dev(_rand((K, M + 4), 41))[:, :M], dev(_rand((K, N + pad), 42))[:, :N], None, 0, C2)
    assert torch.equal(C, C2)


@pytest.mark.parametrize("M,N,K", [(32768, 256, 32), (1000, 70, 4), (77, 300, 64), (5000, 33, 20), (31, 256, 8), (4100, 520, 48)])
def test_gemm_fp32_short_reduction(M, N, K):
    # A B^T with a reduction of classifier length (at most 64): every epilogue, ragged rows and columns
    A = _rand((M, K), 43); Bt = _rand((N, K), 44); bias = _rand(N, 45)
    mask = np.maximum(_rand((M, N), 46), 0.0)
    C = torch.full((M, N + 4), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, 0, C[:, :N])
    prod = oracle.gemm(A, Bt.T.copy())
    assert rel_err(C[:, :N].cpu().numpy(), prod) < TOL_F32
    assert torch.all(C[:, N:] == 7.0)
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), dev(bias), sg.SGNN_RELU, C[:, :N])
    assert rel_err(C[:, :N].cpu().numpy(), np.maximum(prod + bias, 0)) < TOL_F32
    sg.sgnn_gemm(ctx(), False, True, dev(A), dev(Bt), None, 0, C[:, :N], mask=dev(mask))
    assert rel_err(C[:, :N].cpu().numpy(), np.where(mask > 0, prod, 0.0)) < TOL_F32
    assert torch.all(C[:, :N][dev(mask) <= 0] == 0)


def test_gemm_fp32_weight_gradient_shape():
    # dW = T^T dZ of the headline workload: 256 x 256 result, reduction over 32768 rows, split and summed in a fixed order
    K, M, N = 32768, 256, 256
    ctx().reserve(1, 1, 40000, 256)
    At = _rand((K, M), 26); Bm = _rand((K, N), 27)
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, 0, C)
    assert rel_err(C.cpu().numpy(), oracle.gemm(At.T.copy(), Bm)) < TOL_F32
    C2 = torch.zeros_like(C)
    sg.sgnn_gemm(ctx(), True, False, dev(At), dev(Bm), None, 0, C2)
    assert torch.equal(C, C2)


@pytest.mark.parametrize("M,N,K,ldpad", [(5000, 256, 256, 0), (4100, 47, 256, 0), (9000, 172, 128, 4), (4097, 256, 100, 0),
                                         (6000, 256, 47, 1), (4608, 64, 32, 0), (4096, 200, 172, 0), (70000, 256, 256, 0)])
def test_gemm_bf16_tall_operand(M, N, K, ldpad):
    # tall A, small B: the shape of the layer transform and of the feature gradient of a large mini-batch
    # (ldpad: extra columns behind A's rows, holding values that must not enter the product)
    A = _rand((M, K + ldpad), 11); Bm = _rand((K, N), 12); Bt = _rand((N, K), 13); bias = _rand(N, 14)
    Ad = dev(A)[:, :K]
    Ar = oracle.round_bf16(A[:, :K])
    Cfull = torch.full((M, N + 3), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, False, Ad, dev(Bm), dev(bias), sg.SGNN_RELU | sg.SGNN_BF16_MFMA, Cfull[:, :N])
    ref = np.maximum(oracle.gemm(Ar, oracle.round_bf16(Bm)) + bias, 0)
    assert rel_err(Cfull[:, :N].cpu().numpy(), ref) < 1e-4
    assert torch.all(Cfull[:, N:] == 9.0)
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, True, Ad, dev(Bt), None, sg.SGNN_BF16_MFMA, C)
    assert rel_err(C.cpu().numpy(), oracle.gemm(Ar, oracle.round_bf16(Bt).T.copy())) < 1e-4


def test_gemm_bf16_rounding_is_nearest_even():
    # K = 1 against a one: the product is the rounded operand itself
    x = np.concatenate([_rand(4000, 10), np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38], np.float32)])
    A = x.reshape(-1, 1); one = np.ones((1, 1), np.float32)
    C = torch.zeros((len(x), 1), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, False, dev(A), dev(one), None, sg.SGNN_BF16_MFMA, C)
    assert np.array_equal(C.cpu().numpy().astype(np.float64).ravel(), oracle.round_bf16(x))


def test_gemm_strided_operands():
    A = _rand((200, 70), 1); Bm = _rand((64, 50), 2)
    Ad = dev(A)[:, :64]; Bd = dev(Bm)[:, :48]
    Cfull = torch.zeros((200, 52), dtype=torch.float32, device=DEV)
    sg.sgnn_gemm(ctx(), False, False, Ad, Bd, None, 0, Cfull[:, :48])
    assert rel_err(Cfull[:, :48].cpu().numpy(), A[:, :64].astype(np.float64) @ Bm[:, :48]) < TOL_F32
    assert torch.all(Cfull[:, 48:] == 0)


@pytest.mark.parametrize("xform", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d_in,d_out,relu", [(32, 64, True), (64, 8, False), (100, 256, True), (256, 47, False), (602, 256, True)])
def test_layer_forward_backward(sub, d_in, d_out, relu, bf16, xform):
    B, rp, ci, v = sub
    ctx().reserve(B, len(ci), B, max(d_in, d_out), len(ci))
    A = sg.Csr.from_arrays(B, B, rp, ci, v, DEV)
    H = _rand((B, d_in), 1); W = (_rand((d_in, d_out), 2) / np.sqrt(d_in)).astype(np.float32); b = _rand(d_out, 3) * 0.1
    dY = _rand((B, d_out), 4)
    flags = (sg.SGNN_RELU if relu else 0) | (sg.SGNN_BF16_MFMA if bf16 else 0) | (sg.SGNN_XFORM_FIRST if xform else 0)
    tol = TOL_BF16 if bf16 else TOL_F32
    Y = torch.zeros((B, d_out), dtype=torch.float32, device=DEV); T = torch.zeros((B, d_in), dtype=torch.float32, device=DEV)
    sg.sgnn_gcn_fwd(ctx(), A, dev(H), dev(W), dev(b), flags, Y, None if xform else T)
    T_ref, Y_ref = oracle.gcn_fwd(rp, ci, v, H, W, b, relu=relu, bf16=bf16)
    if not xform:
        assert rel_err(T.cpu().numpy(), T_ref) < TOL_F32
    assert rel_err(Y.cpu().numpy(), Y_ref) < tol
    # backward from the oracle's own forward state
    rpT, ciT, vT = oracle.csr_transpose(B, B, rp, ci, v)
    dH_ref, dW_ref, db_ref = oracle.gcn_bwd(rpT, ciT, vT, T_ref, W, Y_ref, dY, relu=relu, bf16=bf16)
    AT = sg.Csr.from_arrays(B, B, rpT, ciT, vT, DEV)
    dH = torch.zeros((B, d_in), dtype=torch.float32, device=DEV)
    dW = torch.zeros((d_in, d_out), dtype=torch.float32, device=DEV); db = torch.zeros(d_out, dtype=torch.float32, device=DEV)
    saved = dev(H) if xform else dev(T_ref, torch.float32)     # transform-first layers keep their input
    sg.sgnn_gcn_bwd(ctx(), AT, saved, dev(W), dev(Y_ref, torch.float32), dev(dY), flags, dH, dW, db)
    assert rel_err(dH.cpu().numpy(), dH_ref) < tol
    assert rel_err(dW.cpu().numpy(), dW_ref) < tol
    assert rel_err(db.cpu().numpy(), db_ref) < TOL_F32
    # first layer: dH skipped, nothing else changes
    dW2 = torch.zeros_like(dW)
    sg.sgnn_gcn_bwd(ctx(), AT, saved, dev(W), dev(Y_ref, torch.float32), dev(dY), flags, None, dW2, None)
    assert torch.equal(dW, dW2)
    # the ReLU backward of the layer below fused into the product that writes dH: zero where H_in <= 0
    Hm = np.maximum(_rand((B, d_in), 5), 0)
    dH3 = torch.full((B, d_in), 7.0, dtype=torch.float32, device=DEV)
    sg.sgnn_gcn_bwd(ctx(), AT, saved, dev(W), dev(Y_ref, torch.float32), dev(dY), flags, dH3, dW2, None, H_in=dev(Hm))
    assert torch.equal(dH3, dH * (dev(Hm) > 0))
    # ... and the other side of that contract: a dY that already carries this layer's mask needs no Y
    if relu:
        dYm = dY * (Y_ref > 0)
        dH4 = torch.zeros_like(dH); dW4 = torch.zeros_like(dW); db4 = torch.zeros_like(db)
        sg.sgnn_gcn_bwd(ctx(), AT, saved, dev(W), None, dev(dYm.astype(np.float32)), flags | sg.SGNN_DY_MASKED, dH4, dW4, db4)
        assert torch.equal(dH4, dH) and torch.equal(dW4, dW)
        # the bias gradient now rides on the weight-gradient product: another (fixed) summation order
        assert rel_err(db4.cpu().numpy(), db_ref) < TOL_F32


def test_backward_uses_the_transpose():
    rp = np.array([0, 2, 3, 6], np.int32); ci = np.array([0, 2, 0, 0, 1, 2], np.int32)
    v = np.array([0.5, -1.0, 2.0, 0.25, 3.0, 1.5], np.float32)
    H = _rand((3, 4), 1); W = _rand((4, 2), 2); R = _rand((3, 2), 3)
    ctx().reserve(3, 6, 3, 4, 6)
    T_ref, Y_ref = oracle.gcn_fwd(rp, ci, v, H, W, None, relu=False)
    rpT, ciT, vT = oracle.csr_transpose(3, 3, rp, ci, v)
    dH_ref, dW_ref, _ = oracle.gcn_bwd(rpT, ciT, vT, T_ref, W, Y_ref, R, relu=False)
    AT = sg.Csr.from_arrays(3, 3, rpT, ciT, vT, DEV)
    dH = torch.zeros((3, 4), dtype=torch.float32, device=DEV); dW = torch.zeros((4, 2), dtype=torch.float32, device=DEV)
    sg.sgnn_gcn_bwd(ctx(), AT, dev(T_ref, torch.float32), dev(W), None, dev(R), 0, dH, dW, None)
    assert rel_err(dH.cpu().numpy(), dH_ref) < TOL_F32 and rel_err(dW.cpu().numpy(), dW_ref) < TOL_F32


def test_softmax_xent_and_gather():
    B, C = 1000, 47
    O = _rand((B, C), 1) * 3; y = np.random.default_rng(2).integers(0, C, B).astype(np.int32)
    ctx().reserve(B, 1, B, C)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV); dO = torch.zeros((B, C), dtype=torch.float32, device=DEV)
    sg.sgnn_softmax_xent(ctx(), dev(O), dev(y), loss, dO)
    l_ref, dO_ref = oracle.softmax_xent(O, y)
    assert abs(loss.item() - l_ref) < TOL_F32 * abs(l_ref) and rel_err(dO.cpu().numpy(), dO_ref) < TOL_F32
    X = _rand((5000, 100), 3); S = np.sort(np.random.default_rng(4).permutation(5000)[:B]).astype(np.int32)
    labels = np.random.default_rng(5).integers(0, C, 5000).astype(np.int32)
    out = torch.zeros((B, 100), dtype=torch.float32, device=DEV); lo = torch.zeros(B, dtype=torch.int32, device=DEV)
    sg.sgnn_gather_rows(ctx(), dev(X), dev(S), B, out, dev(labels), lo)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.gather_rows(X, S))
    assert np.array_equal(lo.cpu().numpy(), oracle.gather_labels(labels, S))
    lo2 = torch.zeros(B, dtype=torch.int32, device=DEV)
    sg.sgnn_gather_rows(ctx(), None, dev(S), B, None, dev(labels), lo2)
    assert torch.equal(lo, lo2)


@pytest.mark.parametrize("B,C", [(1000, 47), (32768, 32), (77, 3), (5000, 172), (4099, 64), (300, 700)])
def test_softmax_xent_with_column_sums(B, C):
    # the column sums of dO (bias gradient of a last layer without activation) from the same pass: every class-count
    # bracket of the kernel (lanes per row, values per lane), ragged row counts, and the plain call unchanged by it
    O = _rand((B, C + 1), 6)[:, :C] * 3; y = np.random.default_rng(7).integers(0, C, B).astype(np.int32)
    ctx().reserve(B, 1, B, max(C, 8))
    loss = torch.zeros(1, dtype=torch.float32, device=DEV); dO = torch.zeros((B, C), dtype=torch.float32, device=DEV)
    cs = torch.full((C,), 9.0, dtype=torch.float32, device=DEV)
    Od = dev(_rand((B, C + 1), 6) * 3)[:, :C]
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss, dO, dO_colsum=cs)
    l_ref, dO_ref = oracle.softmax_xent(O.copy(), y)
    assert abs(loss.item() - l_ref) < TOL_F32 * abs(l_ref) and rel_err(dO.cpu().numpy(), dO_ref) < TOL_F32
    # a column of dO sums values of both signs: the error is measured against the sum of their magnitudes
    assert np.abs(cs.cpu().numpy() - dO_ref.sum(axis=0)).max() < TOL_F32 * np.abs(dO_ref).sum(axis=0).max()
    loss2 = torch.zeros_like(loss); dO2 = torch.zeros_like(dO); cs2 = torch.zeros_like(cs)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, dO2, dO_colsum=cs2)
    assert torch.equal(cs, cs2) and torch.equal(loss, loss2)
    dO3 = torch.zeros_like(dO)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, dO3)
    assert torch.equal(dO, dO3) and torch.equal(loss, loss2)
    with pytest.raises(sg.SgnnError):
        sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, None, dO_colsum=cs2)


@pytest.mark.parametrize("B,C", [(5000, 172), (4099, 64), (300, 700), (32768, 32), (1000, 1024), (77, 16), (1, 48)])
def test_softmax_xent_aligned_rows_and_large_logits(B, C):
    # class counts and leading dimensions that are multiples of four (rows 16-byte aligned), every lanes-per-row bracket,
    # ragged row counts, logits in the hundreds (the label's logit comes from the lane that holds its column)
    O = _rand((B, C + 4), 8)[:, :C] * 5; y = np.random.default_rng(9).integers(0, C, B).astype(np.int32)
    O[::7] *= 40.0                                   # rows with logits in the hundreds
    ctx().reserve(B, 1, B, max(C, 8))
    Od = dev(np.pad(O, ((0, 0), (0, 4))))[:, :C]
    assert Od.stride(0) % 4 == 0
    loss = torch.zeros(1, dtype=torch.float32, device=DEV); dO = torch.zeros((B, C + 4), dtype=torch.float32, device=DEV)[:, :C]
    cs = torch.full((C,), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss, dO, dO_colsum=cs)
    l_ref, dO_ref = oracle.softmax_xent(O.copy(), y)
    assert abs(loss.item() - l_ref) < TOL_F32 * abs(l_ref) and rel_err(dO.cpu().numpy(), dO_ref) < TOL_F32
    assert np.abs(cs.cpu().numpy() - dO_ref.sum(axis=0)).max() < TOL_F32 * np.abs(dO_ref).sum(axis=0).max()
    loss2 = torch.zeros_like(loss); dO2 = torch.zeros_like(dO); cs2 = torch.zeros_like(cs)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, dO2, dO_colsum=cs2)
    assert torch.equal(cs, cs2) and torch.equal(loss, loss2) and torch.equal(dO, dO2)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, None)       # the loss alone
    # dO stored as bfloat16: the same values rounded to nearest even once, and the column sums of what is stored
    dO16 = torch.zeros((B, (C + 31) // 32 * 32), dtype=torch.bfloat16, device=DEV)[:, :C]; cs16 = torch.zeros_like(cs)
    sg.sgnn_softmax_xent(ctx(), Od, dev(y), loss2, dO16, dO_colsum=cs16)
    assert torch.equal(dO16, dO.to(torch.bfloat16)) and torch.equal(loss, loss2)
    stored = dO16.float().cpu().numpy().astype(np.float64)
    assert np.abs(cs16.cpu().numpy() - stored.sum(axis=0)).max() < TOL_F32 * np.abs(stored).sum(axis=0).max()
    assert torch.equal(loss, loss2)


def _run_config(name, steps, fuse_slice, bf16=None, auto_order=True, fuse_relu_bwd=True, bf16_act=False, fuse_loss=False):
    cfg = si.CONFIGS[name]
    bf16 = cfg.bf16_mfma if bf16 is None else bf16
    # inputs are generated with torch on the GPU (integer parts are device independent) and copied
    # to the host for the oracle
    gd = si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=DEV)
    Xd = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=DEV)
    ld = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=DEV)
    weights = si.layer_weights(cfg)
    st = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld,
                    [(W.to(DEV), b.to(DEV)) for W, b in weights], cfg.B, cfg.sampler_seed, bf16=bf16,
                    fuse_slice=fuse_slice, device=DEV, auto_order=auto_order, fuse_relu_bwd=fuse_relu_bwd,
                    bf16_activations=bf16_act, fuse_loss=fuse_loss)
    assert st.fuse_loss == fuse_loss
    g = si.Graph(cfg.N, gd.rowptr.cpu(), gd.colidx.cpu())
    X, labels = Xd.cpu(), ld.cpu()
    wnp = [(W.double().numpy(), b.double().numpy()) for W, b in weights]
    tol = TOL_BF16 if bf16 else TOL_F32
    band = 1e-3 if bf16 else 1e-5
    for t in steps:
        st.step(t)
        torch.cuda.synchronize()
        st.ctx.status()
        args = (cfg.N, g.rowptr.numpy(), g.colidx.numpy(), X.numpy(), labels.numpy(), wnp, cfg.B, cfg.sampler_seed, t)
        ref = oracle.gcn_step(*args, bf16=bf16, tie_band=band, store_bf16=bf16_act)
        nnz = st.A.nnz()
        assert np.array_equal(st.S.cpu().numpy(), ref["S"])
        assert np.array_equal(st.A.rowptr.cpu().numpy(), ref["rowptr"]) and nnz == len(ref["colidx"])
        assert np.array_equal(st.A.colidx.cpu().numpy()[:nnz], ref["colidx"])
        got_val = st.A.val.cpu().numpy()[:nnz].astype(np.float64)
        assert np.all(np.abs(got_val - ref["val"]) <= TOL_VAL * np.abs(ref["val"]))
        assert np.array_equal(st.y_S.cpu().numpy(), ref["y_S"])
        if not fuse_slice:
            assert np.array_equal(st.X_S.cpu().numpy().astype(np.float64), ref["X_S"])
        ties = []
        for l in range(cfg.layers):
            if st.T[l] is not None:      # transform-first layers never form the aggregate
                assert rel_err(st.T[l].float().cpu().numpy(), ref["T"][l]) < tol, ("T", l)
            assert rel_err(st.H[l].float().cpu().numpy(), ref["H"][l + 1]) < tol, ("H", l)
            # the ReLU decision must agree wherever the pre-activation is decidably non-zero
            got_mask = st.H[l].float().cpu().numpy() > 0
            if l < cfg.layers - 1:
                assert np.array_equal(got_mask[~ref["relu_band"][l]], ref["relu_mask"][l][~ref["relu_band"][l]])
            ties.append(got_mask)
        assert abs(st.loss.item() - ref["loss"]) < tol * abs(ref["loss"])
        # inside the undecidable band either mask is correct: the gradients are checked against the
        # oracle evaluated with the decisions the kernels took there
        kw = {}
        if bf16:
            # the loss gradient has an undecidable set as well (rows with large, unsaturated logits, defined by the
            # oracle from its own logits): the device's rows enter there, after being checked against the definition
            # and after the device's logits have been shown to lie within the band of the oracle's
            und = oracle.undecidable_loss_rows(ref["H"][-1], ref["y_S"], LOGIT_BAND, tol)
            O_gpu = st.H[-1].cpu().numpy().astype(np.float64)
            dO_gpu = st.dO.float().cpu().numpy().astype(np.float64)
            _, dO_def = oracle.softmax_xent(O_gpu, ref["y_S"])
            assert rel_err(dO_gpu, dO_def) < (2.0 ** -8 if st.dO.dtype == torch.bfloat16 else TOL_F32)   # as stored
            eps = LOGIT_BAND * np.abs(ref["H"][-1]).max(axis=1)
            assert np.all(np.abs(O_gpu - ref["H"][-1])[und] <= eps[und, None])
            assert und.mean() < 0.1
            if und.any():
                kw = dict(logit_band=LOGIT_BAND, grad_band=tol, dO_ties=dO_gpu)
        if any((ties[l] != ref["relu_mask"][l]).any() for l in range(cfg.layers - 1)) or kw:
            ref = oracle.gcn_step(*args, bf16=bf16, tie_band=band, relu_ties=ties, store_bf16=bf16_act, **kw)
        for l in range(cfg.layers):
            assert rel_err(st.dW[l].cpu().numpy(), ref["dW"][l]) < tol, ("dW", l)
            assert rel_err(st.db[l].cpu().numpy(), ref["db"][l]) < tol, ("db", l)
            if l > 0:
                # with the ReLU backward of layer l-1 fused into the product that writes dH, the buffer holds
                # dH where H_{l-1} > 0 and zero elsewhere (the mask was checked against the oracle's above)
                want = ref["dH"][l] * ties[l - 1] if fuse_relu_bwd else ref["dH"][l]
                assert rel_err(st.dH[l].float().cpu().numpy(), want) < tol, ("dH", l)


@pytest.mark.parametrize("fuse_relu_bwd", [False, True])
@pytest.mark.parametrize("auto_order", [False, True])
@pytest.mark.parametrize("fuse_slice", [False, True])
def test_whole_step_tiny(fuse_slice, auto_order, fuse_relu_bwd):
    _run_config("tiny", [0, 1], fuse_slice, auto_order=auto_order, fuse_relu_bwd=fuse_relu_bwd)


def test_whole_step_with_a_narrowing_first_layer():
    # first layer 32 -> 16 evaluated transform-first straight from the full feature matrix
    # (row_index = S in the forward GEMM and in the weight-gradient GEMM)
    import copy
    cfg = copy.deepcopy(si.CONFIGS["tiny"]); cfg.hidden = 16; cfg.name = "tiny_narrow"
    si.CONFIGS["tiny_narrow"] = cfg
    try:
        _run_config("tiny_narrow", [0], True)
        _run_config("tiny_narrow", [1], False)
    finally:
        del si.CONFIGS["tiny_narrow"]


def test_whole_step_with_narrow_layers_and_a_long_batch():
    # two narrowing layers (32 -> 16 -> 8) over 6000 sampled vertices: both weight gradients are long reductions onto
    # results of at most 16 columns, the first one reading the feature rows through row_index = S
    si.CONFIGS["narrow_long"] = si.Config("narrow_long", 16384, 131072, 32, 16, 2, 8, 6000)
    try:
        _run_config("narrow_long", [0], True)
        _run_config("narrow_long", [1], False)
    finally:
        del si.CONFIGS["narrow_long"]


def test_whole_step_with_a_ragged_feature_width():
    # 100 features into 96 hidden units, transform-first, 4128 sampled vertices: the step pads the features to 128
    # columns, and both products of the first layer gather their rows of X inside the direct-to-LDS kernels
    # (X[S] W_1 by tile row, X[S]^T dP by reduction row, a long reduction split into ranges)
    si.CONFIGS["ragged_wide"] = si.Config("ragged_wide", 16384, 131072, 100, 96, 2, 8, 4128)
    try:
        _run_config("ragged_wide", [0, 1], True)
        _run_config("ragged_wide", [2], False)
    finally:
        del si.CONFIGS["ragged_wide"]


def test_whole_step_with_the_loss_in_the_last_sparse_product():
    # transform-first last layers: O = A (H W) + b, the loss and its gradient from one kernel (sgnn_spmm_xent)
    _run_config("tiny", [0, 3], True, fuse_loss=True)
    _run_config("medium", [1], True, fuse_loss=True)
    _run_config("medium", [2], True, bf16=True, bf16_act=True, fuse_loss=True)


def test_whole_step_tiny_bf16():
    _run_config("tiny", [0], True, bf16=True)


def test_whole_step_medium():
    _run_config("medium", [0, 15], True)


@pytest.mark.parametrize("auto_order", [False, True])
@pytest.mark.parametrize("fuse_relu_bwd", [False, True])
def test_whole_step_bf16_activations_medium(auto_order, fuse_relu_bwd):
    # |S| = 32768: the tall-operand kernel reads and writes the 16-bit activations itself (aggregate-first and
    # transform-first layers, fused and separate ReLU backward)
    _run_config("medium", [3], True, bf16=True, auto_order=auto_order, fuse_relu_bwd=fuse_relu_bwd, bf16_act=True)


@pytest.mark.parametrize("fuse_slice", [False, True])
def test_whole_step_bf16_activations_tiny(fuse_slice):
    # |S| = 1024: every product goes through the fp32 copies in scratch
    _run_config("tiny", [0, 1], fuse_slice, bf16=True, bf16_act=True)
    _run_config("tiny", [2], fuse_slice, bf16=True, bf16_act=True, auto_order=False, fuse_relu_bwd=False)


def test_whole_step_large_bf16():
    # co-purchase-shaped graph at full size: 2.4 M vertices, 124 M stored entries, |S| = 262144
    _run_config("large", [0], True)


def test_whole_step_large_bf16_storage():
    # the same graph in the configuration bench.py times: activations, hand-down gradients and the loss gradient
    # stored as bfloat16 (another sampler counter than the fp32-storage test above)
    _run_config("large", [1], True, bf16_act=True)


def test_whole_step_large_with_the_loss_in_the_last_sparse_product():
    # as above with the loss and its gradient formed in the epilogue of the last sparse product (logits kept, so that
    # the oracle's statement about them can be checked)
    _run_config("large", [2], True, bf16_act=True, fuse_loss=True)


@pytest.mark.parametrize("name,bf16", [("large", True), ("medium", False)])
def test_step_without_logits_is_the_step_with_logits(name, bf16):
    # The launch configuration bench.py times does not write the logits: the same kernels with the stores of O left
    # out.  Loss, loss gradient and every weight and bias gradient must come out bit for bit as with the logits kept
    # (checked against the oracle above).
    cfg = si.CONFIGS[name]
    gd = si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=DEV)
    Xd = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=DEV)
    ld = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=DEV)
    weights = si.layer_weights(cfg)
    got = []
    for keep in (True, False):
        st = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, [(W.to(DEV), b.to(DEV)) for W, b in weights], cfg.B,
                        cfg.sampler_seed, bf16=bf16, fuse_slice=True, device=DEV, bf16_activations=bf16, fuse_loss=True,
                        keep_logits=keep)
        assert st.fuse_loss and st.keep_logits == keep
        st.step(5)
        torch.cuda.synchronize()
        st.ctx.status()
        got.append([st.loss.clone(), st.dO.clone()] + [w.clone() for w in st.dW] + [b.clone() for b in st.db])
        del st
    for a, b in zip(*got):
        assert torch.equal(a, b)


def test_whole_step_dense():
    # social-shaped graph at full size: mean degree about 490, |S| = 65536, 602 input features
    _run_config("dense", [0], True)


def test_whole_step_xlarge_bf16():
    """Citation-shaped graph at full size: 111 M vertices, 3.3 G stored entries, |S| = 2^20, bf16 GEMM
    operands.  The oracle never sees the whole feature matrix: feature rows and labels are a function
    of (seed, vertex), so it regenerates the sampled rows on the host."""
    if torch.cuda.get_device_properties(0).total_memory < 200e9:
        pytest.skip("needs the 288 GB of an MI355X")
    cfg = si.CONFIGS["xlarge"]
    gd = si.config_graph(cfg, device=DEV)
    assert abs((gd.E - cfg.N) / 2 / cfg.undirected_edges - 1.0) < 0.01
    assert cfg.bf16_features
    Xd = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=DEV, dtype=torch.bfloat16)     # 28 GB
    ld = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=DEV)
    weights = si.layer_weights(cfg)
    st = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, [(W.to(DEV), b.to(DEV)) for W, b in weights], cfg.B,
                    cfg.sampler_seed, bf16=True, fuse_slice=True, device=DEV, bf16_activations=True)   # as the benchmark runs it
    st.step(0)
    torch.cuda.synchronize()
    st.ctx.status()
    # oracle side
    S = oracle.sample_uniform(cfg.N, cfg.B, cfg.sampler_seed, 0)
    assert np.array_equal(st.S.cpu().numpy(), S)
    rp, ci = gd.rowptr.cpu().numpy(), gd.colidx.cpu().numpy()
    rpS, ciS, vS = oracle.induced_csr(cfg.N, rp, ci, S)
    del rp, ci
    nnz = st.A.nnz()
    assert nnz == len(ciS) and np.array_equal(st.A.rowptr.cpu().numpy(), rpS)
    assert np.array_equal(st.A.colidx.cpu().numpy()[:nnz], ciS)
    got_val = st.A.val.cpu().numpy()[:nnz].astype(np.float64)
    assert np.all(np.abs(got_val - vS) <= 1e-6 * np.abs(vS))
    St = torch.as_tensor(S.astype(np.int64))
    X_S = si.normal_rows(St, cfg.d_in, cfg.feature_seed, dtype=torch.bfloat16).float().numpy()    # the stored values
    y_S = si.labels_for(St, cfg.classes, cfg.label_seed).numpy()
    assert np.array_equal(st.y_S.cpu().numpy(), y_S)
    wnp = [(W.double().numpy(), b.double().numpy()) for W, b in weights]
    store = bool(getattr(st, "bf16_activations", False))
    band_l = LOGIT_BAND      # accuracy of a logit relative to its row's largest (checked below on the rows it matters for)
    ref = oracle.layers_step(rpS, ciS, vS, X_S, y_S, wnp, bf16=True, tie_band=1e-3, store_bf16=store, logit_band=band_l,
                             grad_band=TOL_BF16)
    Hg = [st.H[l].float().cpu().numpy() for l in range(cfg.layers)]
    ties = [h > 0 for h in Hg]
    for l in range(cfg.layers - 1):
        assert np.array_equal(ties[l][~ref["relu_band"][l]], ref["relu_mask"][l][~ref["relu_band"][l]])
    # The loss gradient.  With 1/p = 106 the logits of hub rows reach the hundreds, a relative 2^-8 between the two
    # sides' logits is an absolute 1 there, and a row whose leading logits are that close gets a different softmax
    # row on each side.  The oracle says which rows those are from ITS OWN logits (undecidable_loss_rows); the
    # device's gradient (checked against the definition on the logits it was computed from, to fp32 accuracy)
    # enters the oracle's backward pass inside that set only, and only after its logits have been shown to lie
    # within the band of the oracle's there; every other row starts from the oracle's own gradient.
    O_gpu = Hg[-1].astype(np.float64)
    dO_gpu = st.dO.float().cpu().numpy().astype(np.float64)
    _, dO_def = oracle.softmax_xent(O_gpu, y_S.astype(np.int32))
    assert rel_err(dO_gpu, dO_def) < (2.0 ** -8 if st.dO.dtype == torch.bfloat16 else TOL_F32)       # as stored
    und = ref["dO_band"]
    O_ref = ref["H"][-1]
    eps = band_l * np.abs(O_ref).max(axis=1)
    row_diff = np.abs(dO_gpu - ref["dO"]).max(axis=1) * cfg.B
    print("undecidable loss rows: %d of %d (%.3f %%); largest own-gradient row difference outside them %.2e, inside %.2e"
          % (und.sum(), cfg.B, 100.0 * und.mean(), row_diff[~und].max(), row_diff[und].max() if und.any() else 0.0), flush=True)
    assert und.mean() < 0.02
    assert np.all(np.abs(O_gpu - O_ref)[und] <= eps[und, None])
    assert row_diff[~und].max() <= TOL_BF16          # decidable rows: the two sides' own gradients agree to the bar
    if any((ties[l] != ref["relu_mask"][l]).any() for l in range(cfg.layers - 1)) or und.any():
        ref = oracle.layers_step(rpS, ciS, vS, X_S, y_S, wnp, bf16=True, tie_band=1e-3, relu_ties=ties, store_bf16=store,
                                 logit_band=band_l, grad_band=TOL_BF16, dO_ties=dO_gpu)
    for l in range(cfg.layers):
        if st.T[l] is not None:
            assert rel_err(st.T[l].float().cpu().numpy(), ref["T"][l]) < TOL_BF16, ("T", l)
        assert rel_err(Hg[l], ref["H"][l + 1]) < TOL_BF16, ("H", l)
        assert rel_err(st.dW[l].cpu().numpy(), ref["dW"][l]) < TOL_BF16, ("dW", l)
        assert rel_err(st.db[l].cpu().numpy(), ref["db"][l]) < TOL_BF16, ("db", l)
        if l > 0:
            # the ReLU backward of layer l-1 is fused into the product that writes dH: the buffer holds dH where
            # H_{l-1} > 0 and zero elsewhere (the mask was checked against the oracle's above)
            assert rel_err(st.dH[l].float().cpu().numpy(), ref["dH"][l] * ties[l - 1]) < TOL_BF16, ("dH", l)
    assert abs(st.loss.item() - ref["loss"]) < TOL_BF16 * abs(ref["loss"])

    # The launch configuration bench.py times: the loss and its gradient in the epilogue of the last sparse product, the
    # logits never written.  Same sampler counter, so the same mini-batch: against the step checked above.
    st2 = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, [(W.to(DEV), b.to(DEV)) for W, b in weights], cfg.B,
                     cfg.sampler_seed, bf16=True, fuse_slice=True, device=DEV, bf16_activations=True, fuse_loss=True,
                     keep_logits=False)
    assert st2.fuse_loss
    st2.step(0)
    torch.cuda.synchronize()
    st2.ctx.status()
    assert torch.equal(st2.S, st.S) and torch.equal(st2.A.colidx[:nnz], st.A.colidx[:nnz])
    assert abs(st2.loss.item() - st.loss.item()) < TOL_F32 * abs(st.loss.item())
    # the same fp32 logits enter both forms of the loss; the stored bfloat16 gradient may differ in its last bit
    assert rel_err(st2.dO.float().cpu().numpy(), dO_gpu) <= 2.0 ** -7
    for l in range(cfg.layers):
        assert rel_err(st2.dW[l].cpu().numpy(), st.dW[l].cpu().numpy()) < 2e-3, ("dW", l)
        assert rel_err(st2.db[l].cpu().numpy(), st.db[l].cpu().numpy()) < 2e-3, ("db", l)
    del st2

    # The full graph as the matrix of a sparse product (evaluation forward): 3.3 G entries, int64 row offsets,
    # bfloat16 features.  The oracle computes sampled output rows one by one: random ones and the longest.
    del st, ref
    torch.cuda.empty_cache()
    E = int(gd.colidx.numel())
    c = sg.Context(0)
    c.reserve(cfg.N, E, cfg.N, cfg.d_in, E)
    A = sg.sgnn_graph_normalized_csr(c, cfg.N, gd.rowptr, gd.colidx)
    assert A.rowptr.dtype == torch.int64 and A.rowptr.data_ptr() == gd.rowptr.data_ptr()
    T = torch.empty((cfg.N, cfg.d_in), dtype=torch.float32, device=DEV)
    sg.sgnn_spmm(c, A, Xd, T)
    c.status()
    deg = gd.rowptr[1:] - gd.rowptr[:-1]
    rows = torch.cat([torch.randint(0, cfg.N, (48,), device=DEV, generator=torch.Generator(device=DEV).manual_seed(3)),
                      torch.topk(deg, 4).indices, torch.tensor([0, cfg.N - 1], device=DEV)])
    lists = [gd.colidx[int(gd.rowptr[v]):int(gd.rowptr[v + 1])].long() for v in rows.tolist()]
    cols_all, inv = torch.unique(torch.cat(lists), return_inverse=True)
    dv = deg[rows].double().cpu().numpy(); du_all = deg[cols_all].double().cpu().numpy()
    lens = np.array([len(x) for x in lists]); rp_s = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ci_s = inv.cpu().numpy().astype(np.int32)
    v_s = (1.0 / np.sqrt(np.repeat(dv, lens) * du_all[ci_s])).astype(np.float32)      # Eq. 3, rounded once like the library's
    X_s = Xd[cols_all].float().cpu().numpy().astype(np.float64)
    want = oracle.spmm(rp_s, ci_s, v_s, X_s)
    got = T[rows].cpu().numpy()
    assert lens.max() > 100000                          # a hub row: cut into pieces, finished by the last of them
    for i in range(len(lens)):
        assert rel_err(got[i], want[i]) < TOL_F32, (int(rows[i]), int(lens[i]))
    c.close()


def test_overlapped_pipeline_matches_single_stream():
    """Building the next mini-batch on a second stream while the current one trains gives bit-identical
    results to the single-stream step (every kernel is deterministic), across more steps than buffers."""
    cfg = si.CONFIGS["tiny"]
    gd = si.rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=DEV)
    Xd = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=DEV)
    ld = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=DEV)
    weights = [(W.to(DEV), b.to(DEV)) for W, b in si.layer_weights(cfg)]
    a = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, weights, cfg.B, cfg.sampler_seed, device=DEV)
    b = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, weights, cfg.B, cfg.sampler_seed, device=DEV, side_dw=True)
    for last in (0, 1, 4, 5):
        steps = list(range(last + 1))
        b.run(steps)
        a.step(last)
        torch.cuda.synchronize()
        assert torch.equal(a.S, b.S) and torch.equal(a.A.rowptr, b.A.rowptr)
        assert torch.equal(a.loss, b.loss)
        for l in range(cfg.layers):
            assert torch.equal(a.dW[l], b.dW[l]) and torch.equal(a.db[l], b.db[l]) and torch.equal(a.H[l], b.H[l])
    b.ctx.status(); b.side_ctx.status()
    # the same pipeline replayed from HIP graphs, several rounds, checked after every replay count
    c = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, weights, cfg.B, cfg.sampler_seed, device=DEV, side_dw=True)
    e = sg.GcnStep(cfg.N, gd.rowptr, gd.colidx, Xd, ld, weights, cfg.B, cfg.sampler_seed, device=DEV)     # weight gradients on the main stream
    for g in (c, e):
        # two steps a graph; the whole cycle in one graph; the side branch forked mid-step or at the step's start
        for spg, fork, counts in ((2, "mid", (2, 4, 6, 10)), (0, "mid", (4, 8, 12)), (0, "start", (4, 8))):
            g.build_graphs(range(4), steps_per_graph=spg, fork=fork)
            for n in counts:
                g.run_graphs(n)
                a.step((n - 1) % 4)
                torch.cuda.synchronize()
                assert torch.equal(a.S, g.S) and torch.equal(a.A.rowptr, g.A.rowptr) and torch.equal(a.loss, g.loss)
                for l in range(cfg.layers):
                    assert torch.equal(a.dW[l], g.dW[l]) and torch.equal(a.db[l], g.db[l]) and torch.equal(a.H[l], g.H[l])
        g.ctx.status(); g.side_ctx.status()


@pytest.mark.parametrize("rows,cols", [(1000, 256), (77, 47), (4100, 32), (5, 1)])
def test_column_sums(rows, cols):
    X = _rand((rows, cols + 2), 31)
    out = torch.full((cols,), 9.0, dtype=torch.float32, device=DEV)
    sg.sgnn_colsum(ctx(), dev(X)[:, :cols], out)
    assert rel_err(out.cpu().numpy(), X[:, :cols].astype(np.float64).sum(axis=0)) < TOL_F32
    out2 = torch.zeros_like(out)
    sg.sgnn_colsum(ctx(), dev(X)[:, :cols], out2)
    assert torch.equal(out, out2)
