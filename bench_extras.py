#!/usr/bin/env python3
"""Measurements of the parts of the method around the headline step, one JSON line each:

  python bench_extras.py --what tail  [--config medium]
      the fused layer tail (RMSNorm + ReLU + dropout + residual, Eqs. 7-10) forward and backward
  python bench_extras.py --what eval  [--config large]
      the full-graph evaluation forward: normalised adjacency of all N vertices (Eq. 3), every layer
  python bench_extras.py --what stages [--config large]
      mini-batch construction stage by stage: sampler (Gkeys/s against the integer ALU), induced CSR
      extraction and the feature slice (GB/s of compulsory traffic against HBM)
  python bench_extras.py --what gemm  [--config medium] [--only TN]
      the dense products of one training step at the configuration's shapes (transform, input
      gradient, weight gradient of every layer: Eqs. 6, 22, 24), each alone, against the MFMA peak
  python bench_extras.py --what shard [--config medium] [--grid 2]
      one GPU's share of the distributed extraction (Algorithm 2): the shard of the mini-batch matrix
      for one row range and one column range of a grid x grid partition, and its transpose

Every figure is measured with HIP events recorded on the launch stream around each kernel; byte
counts are the compulsory ones (each operand once).  The headline benchmark is bench.py.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def _timed(ctx, fn, reps, warm=2):
    """Per-kernel [(kernel, tag, launches, total_ms)] of `reps` calls of fn, after `warm` untimed ones."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ctx.profile(True)
    for _ in range(reps):
        fn()
    recs = ctx.profile_read()
    ctx.profile(False)
    return recs


def _kernels(recs, reps):
    return {"%s %s" % (n, t) if t else n: {"launches_per_call": c / reps, "avg_us": 1e3 * ms / c} for n, t, c, ms in recs}


def bench_tail(cfg, args):
    import torch
    import paper_2604_02651_amd as sg
    dev = "cuda:0"
    Bn, d = cfg.B, cfg.hidden
    ctx = sg.Context(0)
    ctx.reserve(1, 1, 1024, 2048)
    gen = torch.Generator(device=dev).manual_seed(1)
    Z = torch.randn((Bn, d), device=dev, generator=gen)
    R = torch.randn((Bn, d), device=dev, generator=gen)
    gam = torch.rand(d, device=dev, generator=gen) + 0.5
    dY = torch.randn((Bn, d), device=dev, generator=gen)
    Y, dZ = torch.empty_like(Z), torch.empty_like(Z)
    ir = torch.empty(Bn, device=dev)
    dg, db = torch.empty(d, device=dev), torch.empty(d, device=dev)
    q = 0.5

    def fn():
        sg.sgnn_tail_fwd(ctx, Z, gam, 1e-6, R, q, 1, 0, 0, Y, ir)
        sg.sgnn_tail_bwd(ctx, Z, ir, gam, q, 1, 0, 0, dY, dZ, dg, db)
    reps = 20
    recs = _timed(ctx, fn, reps)
    byt = 3.0 * Bn * d * 4          # forward: Z, R in, Y out; backward: Z, dY in, dZ out
    ks = _kernels(recs, reps)
    fwd = next(v for k, v in ks.items() if k.startswith("tail_fwd_kernel"))
    bwd = next(v for k, v in ks.items() if k.startswith("tail_bwd_kernel"))
    ctx.status()
    return {"metric": "fused layer tail (RMSNorm+ReLU+dropout+residual), forward + backward", "unit": "GB/s",
            "value": 2 * byt / ((fwd["avg_us"] + bwd["avg_us"]) * 1e-6) / 1e9, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "%s: %d x %d activations, dropout q = %.1f" % (cfg.name, Bn, d, q)},
            "roofline": {"bound": "hbm", "kernel": "tail_fwd_kernel", "achieved": byt / (fwd["avg_us"] * 1e-6) / 1e9,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": byt / (fwd["avg_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS,
                         "avg_launch_us": fwd["avg_us"], "traffic": None,
                         "tail_bwd_kernel": {"achieved": byt / (bwd["avg_us"] * 1e-6) / 1e9, "avg_launch_us": bwd["avg_us"]}},
            "kernels": ks}


def bench_eval(cfg, args):
    import time
    import torch
    import paper_2604_02651_amd as sg
    import synth_inputs as si
    dev = "cuda:0"
    g = si.config_graph(cfg, device=dev)
    E = int(g.colidx.numel())
    X = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=dev,
                           dtype=torch.bfloat16 if cfg.bf16_features else torch.float32)
    weights = si.layer_weights(cfg, device=dev)
    # fp32 activations of all vertices: when they do not fit one GPU (the largest configuration: 114 GB per
    # N x 256 matrix) only the first aggregation, T = A X over all entries, is run
    first_only = 4.0 * cfg.N * (cfg.d_in + 3 * cfg.hidden) * 4 > 0.6 * torch.cuda.get_device_properties(0).total_memory
    if first_only:
        weights = weights[:1]
    ctx = sg.Context(0)
    dmax = cfg.d_in if first_only else max([cfg.d_in] + [W.shape[1] for W, _ in weights])
    ctx.reserve(cfg.N, E, cfg.N, dmax, E)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    A = sg.sgnn_graph_normalized_csr(ctx, cfg.N, g.rowptr, g.colidx)
    torch.cuda.synchronize()
    build_ms = 1e3 * (time.perf_counter() - t0)
    flags0 = sg.SGNN_BF16_MFMA if cfg.bf16_mfma else 0
    if first_only:
        T0 = torch.empty((cfg.N, cfg.d_in), dtype=torch.float32, device=dev)
        bufs = []
    else:
        bufs = [(torch.empty((cfg.N, W.shape[1]), dtype=torch.float32, device=dev),
                 torch.empty((cfg.N, W.shape[0]), dtype=torch.float32, device=dev)) for W, _ in weights]

    def fn():
        if first_only:
            sg.sgnn_spmm(ctx, A, X, T0)
            return
        H = X
        for l, (W, b) in enumerate(weights):
            # a layer that narrows runs transform-first, as in the training step
            fl = flags0 | (sg.SGNN_RELU if l < len(weights) - 1 else 0) | (sg.SGNN_XFORM_FIRST if W.shape[1] < W.shape[0] else 0)
            sg.sgnn_gcn_fwd(ctx, A, H, W, b, fl, bufs[l][0], bufs[l][1])
            H = bufs[l][0]
    reps = 3
    recs = _timed(ctx, fn, reps, warm=1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    wall_ms = 1e3 * (time.perf_counter() - t0) / reps
    ks = _kernels(recs, reps)
    sp_ms = sum(ms for n, t, c, ms in recs if n == "spmm_main_kernel") / reps
    sp_bytes = sp_gather = 0.0
    for n, t, c, ms in recs:
        if n == "spmm_main_kernel":
            d = int(t.split("d=")[1].split()[0])
            xb = 2 if (cfg.bf16_features and d == cfg.d_in) else 4
            sp_bytes += (c / reps) * (8.0 * E + 4.0 * (cfg.N + 1) + cfg.N * d * (4 + xb))
            sp_gather += (c / reps) * (E * d * float(xb))
    ctx.status()
    return {"metric": "full-graph evaluation forward passes/s", "unit": "passes/s", "value": 1e3 / wall_ms, "ms_per_pass": wall_ms,
            "dtype": "bf16" if cfg.bf16_mfma else "f32", "data": "synthetic",
            "config": {"workload": "%s: R-MAT N=%d, E=%d stored entries, %s over all vertices" %
                                   (cfg.name, cfg.N, E, ("first aggregation A X only, d = %d (the activations of the other layers do "
                                                         "not fit one GPU)" % cfg.d_in) if first_only
                                    else "GCN " + "-".join(map(str, cfg.dims))),
                       "normalised_matrix_and_plan_ms": build_ms},
            "roofline": {"bound": "hbm", "kernel": "spmm_main_kernel (all widths)", "achieved": sp_bytes / (sp_ms * 1e-3) / 1e9,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": sp_bytes / (sp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "ms_per_pass": sp_ms, "traffic": None,
                         "gather_GBps": sp_gather / (sp_ms * 1e-3) / 1e9},
            "kernels": ks}


def bench_stages(cfg, args):
    import torch
    import paper_2604_02651_amd as sg
    import synth_inputs as si
    dev = "cuda:0"
    g = si.config_graph(cfg, device=dev)
    E = int(g.colidx.numel())
    X = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=dev)
    labels = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=dev)
    ctx = sg.Context(0)
    exp = cfg.B + (E - cfg.N) * (cfg.B / cfg.N) * ((cfg.B - 1) / max(cfg.N - 1, 1))
    cap = int(min(E, 2 * exp + 16 * cfg.B + 65536))
    ctx.reserve(cfg.N, E, cfg.B, cfg.d_in, cap)
    W = (cfg.N + 63) // 64
    S = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    bm = torch.empty(W, dtype=torch.int64, device=dev)
    rk = torch.empty(W, dtype=torch.int32, device=dev)
    A = sg.Csr(cfg.B, cfg.B, cap, dev)
    X_S = torch.empty((cfg.B, cfg.d_in), dtype=torch.float32, device=dev)
    y_S = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    reps = 8
    steps = iter(range(10 ** 6))
    rec_s = _timed(ctx, lambda: sg.sgnn_sample_uniform(ctx, cfg.N, cfg.B, cfg.sampler_seed, next(steps), S, bm, rk), reps)
    sg.sgnn_sample_uniform(ctx, cfg.N, cfg.B, cfg.sampler_seed, 0, S, bm, rk)
    nnz = sg.sgnn_induced_csr(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, A, want_nnz=True)
    Sl = S.long()
    sumdeg = int((g.rowptr[Sl + 1] - g.rowptr[Sl]).sum().item())
    rec_i = _timed(ctx, lambda: sg.sgnn_induced_csr(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, A), reps)
    rec_g = _timed(ctx, lambda: sg.sgnn_gather_rows(ctx, X, S, cfg.B, X_S, labels, y_S), reps)
    us = lambda recs, pred=lambda n: True: 1e3 * sum(ms for n, _, _, ms in recs if pred(n)) / reps
    t_s, t_g = us(rec_s), us(rec_g)
    t_i = us(rec_i, lambda n: n.startswith("induced"))       # without the SpMM plan of the new matrix
    t_plan = us(rec_i, lambda n: n.startswith("spmm_plan"))
    # sampler: three passes over N/2 Philox blocks of about 100 integer lane-operations each
    lane_ops = 3.0 * (cfg.N / 2.0) * 100.0
    alu_peak = 256 * 4 * 16 * 2.4e9                            # lanes x clock: one 32-bit integer operation per lane and cycle
    ext_bytes = 4.0 * sumdeg + 16.0 * cfg.B + 8.0 * nnz + 4.0 * (cfg.B + 1)
    sl_bytes = 2.0 * cfg.B * cfg.d_in * 4 + 8.0 * cfg.B
    ctx.status()
    return {"metric": "mini-batch construction (sample + induced CSR + slice)", "unit": "us", "value": t_s + t_i + t_plan + t_g,
            "higher_is_better": False, "dtype": "integer keys and indices, f32 values", "data": "synthetic",
            "config": {"workload": "%s: R-MAT N=%d, E=%d stored entries, |S|=%d, d_in=%d" % (cfg.name, cfg.N, E, cfg.B, cfg.d_in),
                       "sum_deg_S": sumdeg, "induced_entries": nnz},
            "sampler": {"us": t_s, "Gkeys_per_s": cfg.N / (t_s * 1e-6) / 1e9, "bound": "alu",
                        "achieved": lane_ops / (t_s * 1e-6) / 1e12, "peak": alu_peak / 1e12, "unit": "T lane-ops/s",
                        "frac": lane_ops / (t_s * 1e-6) / alu_peak},
            "induced_csr": {"us": t_i, "plan_us": t_plan, "bound": "hbm", "algorithmic_bytes": ext_bytes,
                            "achieved": ext_bytes / (t_i * 1e-6) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": ext_bytes / (t_i * 1e-6) / 1e9 / PEAK_HBM_GBS},
            "slice": {"us": t_g, "bound": "hbm", "algorithmic_bytes": sl_bytes, "achieved": sl_bytes / (t_g * 1e-6) / 1e9,
                      "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": sl_bytes / (t_g * 1e-6) / 1e9 / PEAK_HBM_GBS},
            "kernels": {"sampler": _kernels(rec_s, reps), "induced": _kernels(rec_i, reps), "slice": _kernels(rec_g, reps)}}


def bench_gemm(cfg, args):
    """Every dense product of a step of the aggregate-first / transform-first layer stack, alone."""
    import torch
    import paper_2604_02651_amd as sg
    dev = "cuda:0"
    Bn, dims = cfg.B, cfg.dims
    ctx = sg.Context(0)
    ctx.reserve(1, 1, Bn, max(dims))
    flags = sg.SGNN_BF16_MFMA if cfg.bf16_mfma else 0
    peak = 2500.0 if cfg.bf16_mfma else 157.3
    gen = torch.Generator(device=dev).manual_seed(1)
    shapes = []          # (name, trans_a, trans_b, M, N, K, masked)
    for l in range(cfg.layers):
        di, do = dims[l], dims[l + 1]
        shapes.append(("NN layer %d transform" % l, False, False, Bn, do, di, False))
        if l > 0:
            shapes.append(("NT layer %d input gradient" % l, False, True, Bn, di, do, do < di))
        shapes.append(("TN layer %d weight gradient" % l, True, False, di, do, Bn, False))
    if args.only:
        shapes = [sh for sh in shapes if sh[0].startswith(args.only)]
    out, reps = [], 20
    for name, ta, tb, M, N, K, masked in shapes:
        A = torch.randn((K, M) if ta else (M, K), device=dev, generator=gen)
        Bm = torch.randn((N, K) if tb else (K, N), device=dev, generator=gen)
        Cm = torch.empty((M, N), device=dev)
        mask = torch.randn((M, N), device=dev, generator=gen) if masked else None
        recs = _timed(ctx, lambda: sg.sgnn_gemm(ctx, ta, tb, A, Bm, None, flags, Cm, mask=mask), reps)
        us = sum(ms for _, _, _, ms in recs) * 1e3 / reps
        main_us = sum(ms for n, _, _, ms in recs if n == "gemm_kernel") * 1e3 / reps
        fl = 2.0 * M * N * K
        byt = 4.0 * (M * K + K * N + M * N * (2 if masked else 1))
        out.append({"product": name, "M": M, "N": N, "K": K, "us": us, "gemm_kernel_us": main_us,
                    "TFLOP/s": fl / (us * 1e-6) / 1e12, "frac_of_mfma_peak": fl / (us * 1e-6) / 1e12 / peak,
                    "compulsory_GB/s": byt / (us * 1e-6) / 1e9, "kernels": _kernels(recs, reps)})
        del A, Bm, Cm, mask
    ctx.status()
    tot_fl = sum(2.0 * o["M"] * o["N"] * o["K"] for o in out)
    tot_us = sum(o["us"] for o in out)
    return {"metric": "dense products of one training step, each alone (event-timed, launch floor of about 6 us each included)",
            "unit": "TFLOP/s", "value": tot_fl / (tot_us * 1e-6) / 1e12, "us_per_step": tot_us,
            "dtype": "bf16" if cfg.bf16_mfma else "f32", "data": "synthetic",
            "config": {"workload": "%s: |S| = %d, widths %s" % (cfg.name, Bn, "-".join(str(d) for d in dims))},
            "roofline": {"bound": "mfma", "achieved": tot_fl / (tot_us * 1e-6) / 1e12, "peak": peak, "unit": "TFLOP/s",
                         "frac": tot_fl / (tot_us * 1e-6) / 1e12 / peak, "traffic": None},
            "products": out}


def bench_shard(cfg, args):
    import torch
    import paper_2604_02651_amd as sg
    import synth_inputs as si
    dev = "cuda:0"
    g = si.config_graph(cfg, device=dev)
    E = int(g.colidx.numel())
    G = args.grid
    ctx = sg.Context(0)
    cap = int(min(E, 4 * (E * (cfg.B / cfg.N) ** 2 + cfg.B) + 65536))
    ctx.reserve(cfg.N, E, cfg.B, 8, cap)
    W = (cfg.N + 63) // 64
    S = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    bm = torch.empty(W, dtype=torch.int64, device=dev)
    rk = torch.empty(W, dtype=torch.int32, device=dev)
    sg.sgnn_sample_uniform(ctx, cfg.N, cfg.B, cfg.sampler_seed, 0, S, bm, rk)
    full = sg.Csr(cfg.B, cfg.B, cap, dev)
    nnz_full = sg.sgnn_induced_csr(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, full, want_nnz=True)
    # the shard in the middle of the grid: rows of block G//2, columns of block G//2 - 1 (off the diagonal, so
    # the transpose is a different matrix)
    cut = [cfg.N * i // G for i in range(G + 1)]
    r0, r1 = cut[G // 2], cut[G // 2 + 1]
    c0, c1 = cut[max(G // 2 - 1, 0)], cut[max(G // 2 - 1, 0) + 1]
    A = sg.Csr(cfg.B, cfg.B, cap, dev)
    AT = sg.Csr(cfg.B, cfg.B, cap, dev)
    nnz = sg.sgnn_induced_csr_range(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, r0, r1, c0, c1, A, want_nnz=True)
    reps = 10
    rec_full = _timed(ctx, lambda: sg.sgnn_induced_csr(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, full), reps)
    rec_sh = _timed(ctx, lambda: sg.sgnn_induced_csr_range(ctx, cfg.N, g.rowptr, g.colidx, None, S, cfg.B, bm, rk, r0, r1, c0, c1, A), reps)
    rec_tr = _timed(ctx, lambda: sg.sgnn_csr_transpose(ctx, A, AT), reps)
    us = lambda recs: 1e3 * sum(ms for _, _, _, ms in recs) / reps
    ctx.status()
    return {"metric": "shard of the mini-batch matrix + its transpose (one GPU's share of Algorithm 2)", "unit": "us",
            "value": us(rec_sh) + us(rec_tr), "higher_is_better": False, "dtype": "int32 indices, f32 values", "data": "synthetic",
            "config": {"workload": "%s: R-MAT N=%d, E=%d stored entries, |S|=%d, grid %d x %d, rows [%d,%d) x columns [%d,%d)" %
                                   (cfg.name, cfg.N, E, cfg.B, G, G, r0, r1, c0, c1),
                       "shard_entries": nnz, "whole_matrix_entries": nnz_full},
            "shard_extraction_us": us(rec_sh), "transpose_us": us(rec_tr), "whole_matrix_extraction_us": us(rec_full),
            "kernels": {"shard": _kernels(rec_sh, reps), "transpose": _kernels(rec_tr, reps), "whole": _kernels(rec_full, reps)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--what", required=True, choices=["tail", "eval", "shard", "stages", "gemm"])
    ap.add_argument("--config", default=None, help="tiny | medium | large | dense | xlarge (default: medium; eval and stages: large)")
    ap.add_argument("--grid", type=int, default=2, help="shard: the matrix is cut into grid x grid shards")
    ap.add_argument("--only", default="", help="gemm: only the products whose name starts with this (NN, NT, TN)")
    args = ap.parse_args()
    import torch
    import synth_inputs as si
    if not torch.cuda.is_available():
        print("bench_extras: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfg = si.CONFIGS[args.config or ("large" if args.what in ("eval", "stages") else "medium")]
    out = {"tail": bench_tail, "eval": bench_eval, "shard": bench_shard, "stages": bench_stages, "gemm": bench_gemm}[args.what](cfg, args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
