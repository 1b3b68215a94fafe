#!/usr/bin/env python3
"""Benchmark of the mini-batch GCN hot path on one MI355X.

One "step" is one pass of the whole path over one mini-batch: uniform vertex sample -> induced
normalised CSR -> slice -> L GCN layers forward -> cross-entropy -> L layers backward, every
stage in libsgnn's HIP kernels, inputs resident in HBM before the clock starts.

Prints ONE JSON line: throughput in steps/s, the roofline figure of the kernel that takes the
most time (measured with HIP events recorded on the launch stream, in a second pass over the
same steps so that event overhead does not touch the throughput figure), and the CPU oracle
timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "sampled GCN mini-batch steps/sec (fwd+bwd)"
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=160)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", default="medium", help="tiny | medium | large | dense | xlarge (medium is the headline workload)")
    ap.add_argument("--workload", default="gcn", choices=["gcn", "model"],
                    help="gcn: the plain GCN stack of the configuration (the headline); model: the paper's complete model "
                         "(input projection, residual layers with RMSNorm / ReLU / dropout, output head, Adam) at the "
                         "configuration's sizes - an extra measurement, not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fuse-slice", action="store_true")
    ap.add_argument("--no-fuse-relu-bwd", action="store_true",
                    help="separate ReLU-backward pass instead of masking inside the product that writes the input gradient")
    ap.add_argument("--side-dw", action="store_true",
                    help="weight-gradient GEMMs on the second stream, concurrent with the rest of the backward pass "
                         "(default: on the main stream - measured 1.3 % faster since the GEMM epilogues were vectorised)")
    ap.add_argument("--fork", default="mid", choices=["mid", "start"],
                    help="where a captured step forks the next mini-batch's construction: after its first layer, "
                         "rejoining before its last backward call (mid), or around the whole step (start)")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of replaying HIP graphs")
    ap.add_argument("--no-overlap", action="store_true",
                    help="everything on one stream (default: the next mini-batch is sampled on a second stream while this one trains)")
    ap.add_argument("--cpu-steps", type=int, default=0, help="oracle steps to time (0 = pick by config)")
    ap.add_argument("--breakdown", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB copy kernel five times (reference point for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def gemm_flops(tag: str) -> float:
    # tag: "NN 128x128 32768x256x256 f32"
    dims = tag.split()[2].split("x")
    return 2.0 * float(dims[0]) * float(dims[1]) * float(dims[2])


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the single-GPU hot path; --gpus N with N > 1 is not supported "
              "(no collectives are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2604_02651_amd as sg
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    cfg = si.CONFIGS[args.config]
    g = si.config_graph(cfg, device=dev)
    model = args.workload == "model"
    X = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=dev,
                           dtype=torch.bfloat16 if cfg.bf16_features and not model else torch.float32)
    labels = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=dev)
    weights = si.layer_weights(cfg, device=dev)
    if model:
        d_h = cfg.hidden
        n_layers = max(cfg.layers - 1, 1)
        params = {"W_in": si.glorot_uniform(cfg.d_in, d_h, 100, device=dev).contiguous(),
                  "layers": [(si.glorot_uniform(d_h, d_h, 110 + l, device=dev).contiguous(), torch.ones(d_h, device=dev))
                             for l in range(n_layers)],
                  "W_out": si.glorot_uniform(d_h, cfg.classes, 130, device=dev).contiguous()}
        st = sg.ScaleGnnModel(cfg.N, g.rowptr, g.colidx, X, labels, params, cfg.B, sampler_seed=cfg.sampler_seed, drop_q=0.1,
                              drop_seed=1, bf16=cfg.bf16_mfma, optimizer="adam", lr=1e-3, device=dev)
    else:
        st = sg.GcnStep(cfg.N, g.rowptr, g.colidx, X, labels, weights, cfg.B, cfg.sampler_seed, bf16=cfg.bf16_mfma,
                        fuse_slice=not args.no_fuse_slice, device=dev, fuse_relu_bwd=not args.no_fuse_relu_bwd,
                        side_dw=args.side_dw)
    period = max(cfg.steps, 1)   # the configuration's mini-batches: consecutive sampler counters

    use_graph = not args.no_graph and not args.no_overlap and period % 2 == 0 and not model    # the model is launched eagerly
    if use_graph:
        whole = args.steps % period == 0 and args.warmup % period == 0
        st.build_graphs(range(period), steps_per_graph=0 if whole else 2, fork=args.fork)
        if not whole and (args.steps % 2 or args.warmup % 2):
            print("bench.py: with HIP graphs --steps and --warmup must be even", file=sys.stderr)
            sys.exit(2)

    def run(n):
        if args.no_overlap:
            for i in range(n):
                st.step(i % period)
        elif use_graph and not model:
            st.run_graphs(n)
        else:
            st.run([i % period for i in range(n)])

    run(args.warmup)
    torch.cuda.synchronize()
    st.ctx.status()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st.ctx.status()
    steps_per_s = args.steps / elapsed
    # the same K steps on a single stream, for reference
    t1 = time.perf_counter()
    for i in range(args.steps):
        st.step(i % period)
    torch.cuda.synchronize()
    single_stream_steps_per_s = args.steps / (time.perf_counter() - t1)

    # ---- per-kernel pass: the same steps with every launch bracketed by events on its stream ----
    nprof = min(args.steps, period)
    st.ctx.profile(True)
    nnz_total = 0
    for i in range(nprof):
        st.step(i % period)
    recs = st.ctx.profile_read()
    st.ctx.profile(False)
    for i in range(nprof):     # entry counts of those steps, for the byte figures of the sparse kernels
        if model:
            st.minibatch(i % period)
        else:
            st.sample(i % period); st.induce()
        nnz_total += st.A.nnz()
    nnz_avg = nnz_total / nprof
    groups = {}
    for name, tag, calls, ms in recs:
        key = name   # one group per kernel symbol, as rocprofv3 lists them
        if name == "gemm_kernel":
            p = tag.split()
            key = "gemm_kernel<%s,%s,%s>" % (p[1], p[0], p[3])
        elif name == "spmm_main_kernel":
            key = name + tag.split()[2]
        gq = groups.setdefault(key, {"calls": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        gq["calls"] += calls
        gq["ms"] += ms
        if name == "gemm_kernel":
            gq["flops"] += gemm_flops(tag) * calls
        elif name == "gemm_skinny_bf16_kernel":
            # tall operand streamed once, small operand resident: bound by reading A and writing C
            m_, n_, k_ = (float(x) for x in tag.split()[2].split("x"))
            gq["bytes"] += calls * 4.0 * (m_ * k_ + m_ * n_ + k_ * n_)
        elif name == "spmm_main_kernel":
            d = int(tag.split("d=")[1].split()[0])
            # compulsory traffic: CSR once, every input row once, the output once
            gq["bytes"] += calls * (8.0 * nnz_avg + 4.0 * (cfg.B + 1) + 2.0 * cfg.B * d * 4)
    total_ms = sum(v["ms"] for v in groups.values())
    dom_name, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
    sp = [v for k, v in groups.items() if k.startswith("spmm_main_kernel")]
    sparse_ms, sparse_bytes = sum(v["ms"] for v in sp), sum(v["bytes"] for v in sp)
    if args.breakdown:
        for name, tag, calls, ms in recs:
            if name.startswith("spmm") or name.startswith("gemm"):
                print("  %-24s %-40s calls %3d  avg us %8.2f" % (name, tag, calls, 1e3 * ms / calls), file=sys.stderr)
        for k, v in sorted(groups.items(), key=lambda kv: -kv[1]["ms"]):
            print("%-44s calls/step %5.1f  us/step %9.2f  avg us %8.2f" %
                  (k, v["calls"] / nprof, 1e3 * v["ms"] / nprof, 1e3 * v["ms"] / v["calls"]), file=sys.stderr)
        print("sum of kernel time per step: %.1f us; wall per step: %.1f us" % (1e3 * total_ms / nprof, 1e6 / steps_per_s),
              file=sys.stderr)
    if dom["flops"] > 0:
        dt = "bf16" if dom_name.endswith("bf16>") else "f32"
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                    "frac": achieved / PEAK_TFLOPS[dt], "traffic": None}
    else:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9 if dom["bytes"] > 0 else 0.0
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    # HBM bytes per launch of that kernel from the committed counter summary (rocprofv3 --pmc
    # FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of known size), when it covers this workload
    tpath = os.path.join(ROOT, "profiles", "step_%s_hbm_traffic.txt" % cfg.name)
    if os.path.exists(tpath):
        for line in open(tpath):
            w = line.split()
            if len(w) == 3 and w[0] == "traffic" and w[1] == dom_name:
                roofline["traffic"] = float(w[2])
    roofline["kernel"] = dom_name
    roofline["avg_launch_us"] = 1e3 * dom["ms"] / dom["calls"]
    roofline["launches_per_step"] = dom["calls"] / nprof
    roofline["share_of_kernel_time"] = dom["ms"] / total_ms if total_ms > 0 else None
    # the sparse products as a whole (all widths), the other large group
    roofline["spmm_all_widths"] = {"bound": "hbm", "achieved": sparse_bytes / (sparse_ms * 1e-3) / 1e9 if sparse_ms > 0 else 0.0,
                                   "peak": PEAK_HBM_GBS, "unit": "GB/s", "us_per_step": 1e3 * sparse_ms / nprof}

    out = {
        "metric": METRIC, "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.bf16_mfma else "f32", "data": "synthetic",
        "config": {"workload": "%s: R-MAT N=%d, E=%d stored entries, |S|=%d, %s, %d mini-batches (sampler "
                               "counters 0..%d)" % (cfg.name, cfg.N, g.E, cfg.B,
                                                     ("complete model %d-[%d x %d]-%d with dropout 0.1 and Adam"
                                                      % (cfg.d_in, cfg.hidden, max(cfg.layers - 1, 1), cfg.classes)) if model
                                                     else "GCN " + "-".join(map(str, cfg.dims)), period, period - 1),
                   "fuse_slice": not args.no_fuse_slice, "fuse_relu_bwd": not args.no_fuse_relu_bwd, "side_stream_dw": args.side_dw and not args.no_overlap,
                   "overlap_sampling": not args.no_overlap, "hip_graph": use_graph,
                   "single_stream_steps_per_s": single_stream_steps_per_s, "avg_induced_entries": nnz_avg,
                   "kernel_time_us_per_step": 1e3 * total_ms / nprof},
        "roofline": roofline,
    }

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            sg.sgnn_copy_f32(st.ctx, src, dst)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline and not model:
        import oracle
        rp, ci = g.rowptr.cpu().numpy(), g.colidx.cpu().numpy()
        Xh, lh = X.float().cpu().numpy(), labels.cpu().numpy()
        wnp = [(W.double().cpu().numpy(), b.double().cpu().numpy()) for W, b in weights]
        nsteps = args.cpu_steps or {"tiny": 50, "medium": 8}.get(cfg.name, 1)
        oracle.gcn_step(cfg.N, rp, ci, Xh, lh, wnp, min(cfg.B, 1024), cfg.sampler_seed, 0, bf16=cfg.bf16_mfma)  # warm-up
        c0 = time.perf_counter()
        for t in range(nsteps):
            oracle.gcn_step(cfg.N, rp, ci, Xh, lh, wnp, cfg.B, cfg.sampler_seed, t % period, bf16=cfg.bf16_mfma)
        cpu_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": nsteps / cpu_s, "unit": "steps/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d whole steps (sampler counters 0..%d) of the same workload, %.1f s"
                                         % (nsteps, nsteps - 1, cpu_s)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
