#!/usr/bin/env python3
"""Benchmark of the mini-batch GCN hot path on one MI355X.

One "step" is one pass of the whole path over one mini-batch: uniform vertex sample -> induced
normalised CSR -> slice -> L GCN layers forward -> cross-entropy -> L layers backward, every
stage in libsgnn's HIP kernels, inputs resident in HBM before the clock starts.  Consecutive
steps use consecutive sampler counters (t = 0, 1, 2, ...): no two timed steps of a run share a
mini-batch unless the run is longer than the cycle of captured steps.

Prints ONE JSON line: throughput in steps/s of the headline workload (the largest configuration
that fits one GPU), the roofline figure of the kernel that takes the most time (measured with HIP
events recorded on the launch stream, in a second pass over the same steps so that event overhead
does not touch the throughput figure), the CPU oracle timed on the host cores on a bounded sample
of the same workload, and - as sub-objects under "other_workloads" - the same measurement on
further configurations (fp32 end to end; fp32-stored features).
"""
from __future__ import annotations

import argparse
import gc
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
T_START = time.perf_counter()


def log(msg):
    print("[bench %6.1f s] %s" % (time.perf_counter() - T_START, msg), file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="xlarge",
                    help="tiny | medium | large | dense | xlarge (xlarge, the largest configuration that fits one GPU, "
                         "is the headline workload)")
    ap.add_argument("--extras", default="auto",
                    help="comma-separated further workloads reported as sub-objects: dense, large, medium, tiny, "
                         "xlarge_f32_features; 'auto' = dense,xlarge_f32_features with the xlarge headline, none otherwise; "
                         "'none' = no sub-objects")
    ap.add_argument("--workload", default="gcn", choices=["gcn", "model"],
                    help="gcn: the plain GCN stack of the configuration (the headline); model: the paper's complete model "
                         "(input projection, residual layers with RMSNorm / ReLU / dropout, output head, Adam) at the "
                         "configuration's sizes - an extra measurement, not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fuse-slice", action="store_true")
    ap.add_argument("--no-fuse-relu-bwd", action="store_true",
                    help="separate ReLU-backward pass instead of masking inside the product that writes the input gradient")
    ap.add_argument("--side-dw", action="store_true",
                    help="weight-gradient GEMMs on the second stream, concurrent with the rest of the backward pass")
    ap.add_argument("--fork", default="mid", choices=["mid", "start"],
                    help="where a captured step forks the next mini-batch's construction: after its first layer, "
                         "rejoining before its last backward call (mid), or around the whole step (start)")
    ap.add_argument("--graph", default="auto", choices=["auto", "on", "off"],
                    help="replay HIP graphs of the overlapped pipeline (auto: where a step is short enough to be launch bound)")
    ap.add_argument("--no-graph", action="store_true", help="same as --graph off")
    ap.add_argument("--no-overlap", action="store_true",
                    help="everything on one stream (default: the next mini-batch is sampled on a second stream while this one trains)")
    ap.add_argument("--fuse-loss", choices=["auto", "off", "keep-logits", "drop-logits"], default="auto",
                    help="last layer: the loss and its gradient in the epilogue of the sparse product that forms the logits; "
                         "drop-logits does not write the logits at all, off forms the loss in a kernel of its own; auto (default): "
                         "drop-logits where a mini-batch row is expected to hold fewer than 32 entries, off for dense-degree "
                         "mini-batches (there the product is bound by its gathers and the epilogue's arithmetic comes on top)")
    ap.add_argument("--fp32-loss-grad", action="store_true", help="keep the loss gradient dO in fp32 (default: bfloat16 with the activations)")
    ap.add_argument("--fp32-activations", action="store_true",
                    help="with bf16 GEMM operands, keep the forward activations in fp32 storage (default: bf16 storage)")
    ap.add_argument("--cpu-seconds", type=float, default=25.0, help="target amount of oracle work to time")
    ap.add_argument("--breakdown", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB copy kernel five times (reference point for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--profile-steps-only", type=int, default=0,
                    help="run only this many single-stream steps after the warm-up and print no oracle leg "
                         "(the form the rocprofv3 summaries under profiles/ are made with)")
    return ap.parse_args()


def gemm_flops(tag: str) -> float:
    # tag: "NN 128x128 32768x256x256 f32"
    dims = tag.split()[2].split("x")
    return 2.0 * float(dims[0]) * float(dims[1]) * float(dims[2])


def make_inputs(si, torch, cfg, dev, feature_dtype, graph=None):
    g = graph if graph is not None else si.config_graph(cfg, device=dev)
    log("%s: graph ready (N=%d, E=%d)" % (cfg.name, cfg.N, g.E))
    X = si.normal_features(cfg.N, cfg.d_in, cfg.feature_seed, device=dev, dtype=feature_dtype)
    labels = si.uniform_labels(cfg.N, cfg.classes, cfg.label_seed, device=dev)
    weights = si.layer_weights(cfg, device=dev)
    log("%s: features (%s) / labels / weights ready" % (cfg.name, str(feature_dtype).replace("torch.", "")))
    return g, X, labels, weights


def cycle_length(steps: int) -> int:
    """Number of distinct consecutive mini-batches captured in one HIP graph (even)."""
    if steps % 16 == 0:
        return 16
    if steps <= 64:
        return max(steps - steps % 2, 2)
    return 16


def measure(args, sg, si, torch, cfg, g, X, labels, weights, use_graph_req: str, label: str):
    """Throughput of `args.steps` steps after `args.warmup`, and the per-kernel pass.  Returns
    (fields of the JSON line, the step object)."""
    dev = "cuda:0"
    model = args.workload == "model"
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
        kw = {}
        if "bf16_activations" in sg.GcnStep.__init__.__code__.co_varnames:
            kw["bf16_activations"] = cfg.bf16_mfma and not args.fp32_activations
        if args.fp32_loss_grad:
            kw["bf16_loss_grad"] = False
        fuse_loss = args.fuse_loss
        if fuse_loss == "auto":     # expected entries of a mini-batch row: (E / N) (B / N)
            fuse_loss = "drop-logits" if float(g.E) * cfg.B / (float(cfg.N) * cfg.N) < 32.0 else "off"
        if fuse_loss != "off":
            kw["fuse_loss"] = True
            kw["keep_logits"] = fuse_loss != "drop-logits"
        st = sg.GcnStep(cfg.N, g.rowptr, g.colidx, X, labels, weights, cfg.B, cfg.sampler_seed, bf16=cfg.bf16_mfma,
                        fuse_slice=not args.no_fuse_slice, device=dev, fuse_relu_bwd=not args.no_fuse_relu_bwd,
                        side_dw=args.side_dw, **kw)
    K, W = args.steps, args.warmup

    if args.profile_steps_only:
        for t in range(W):
            st.step(t)
        torch.cuda.synchronize()
        for t in range(args.profile_steps_only):
            st.step(W + t)
        torch.cuda.synchronize()
        st.ctx.status()
        return None, st

    # launch-bound steps (a few hundred microseconds) gain from graph replay; long steps do not
    launch_bound = cfg.B <= 65536 and cfg.name != "dense"
    use_graph = (not model and not args.no_overlap and K >= 2 and
                 (use_graph_req == "on" or (use_graph_req == "auto" and launch_bound)))
    cyc = cycle_length(K) if use_graph else 0
    if use_graph:
        st.build_graphs(range(cyc), steps_per_graph=0, fork=args.fork)     # counters 0 .. cyc-1 in one graph
    n_graph = (K // cyc) * cyc if use_graph else 0

    def eager(ts):
        if args.no_overlap:
            for t in ts:
                st.step(t)
        else:
            st.run(list(ts))

    # warm-up: W eager steps (they also build the second stream's buffers), plus one untimed replay of the graph
    eager(range(W))
    if use_graph:
        st.run_graphs(cyc)
    torch.cuda.synchronize()
    st.ctx.status()
    t0 = time.perf_counter()
    if use_graph:
        st.run_graphs(n_graph)                       # counters 0 .. cyc-1, round and round
    if n_graph < K:
        eager(range(n_graph, K))                     # the remainder, launched from the host
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st.ctx.status()
    steps_per_s = K / elapsed
    # the same K steps on a single stream, for reference
    t1 = time.perf_counter()
    for t in range(K):
        st.step(t)
    torch.cuda.synchronize()
    single_stream_steps_per_s = K / (time.perf_counter() - t1)
    log("%s: %.1f steps/s (single stream %.1f)" % (label, steps_per_s, single_stream_steps_per_s))

    # ---- per-kernel pass: the same steps with every launch bracketed by events on its stream ----
    nprof = min(K, 16)
    st.ctx.profile(True)
    for t in range(nprof):
        st.step(t)
    recs = st.ctx.profile_read()
    st.ctx.profile(False)
    nnz_total = 0
    for t in range(nprof):     # entry counts of those steps, for the byte figures of the sparse kernels
        if model:
            st.minibatch(t)
        else:
            st.sample(t); st.induce()
        nnz_total += st.A.nnz()
    nnz_avg = nnz_total / nprof
    groups = {}
    for name, tag, calls, ms in recs:
        key = name   # one group per kernel symbol, as rocprofv3 lists them
        if name == "gemm_kernel":
            p = tag.split()
            key = "gemm_kernel<%s,%s,%s>" % (p[1], p[0], p[3])
        elif name == "spmm_main_kernel":
            # the instantiation with the loss in its epilogue (tag: "... dO=<bytes>") is a kernel symbol of its own
            key = name + (tag.split()[2][:-1] + ",xent>" if " dO=" in tag else tag.split()[2])
        gq = groups.setdefault(key, {"calls": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        gq["calls"] += calls
        gq["ms"] += ms
        if name in ("gemm_kernel", "gemm_direct_kernel"):
            gq["flops"] += gemm_flops(tag) * calls
        elif name == "gemm_skinny_bf16_kernel":
            # tall operand streamed once, small operand resident: bound by reading A and writing C.
            # tag: "NN|NT skinny MxNxK bf16 [a=<bytes>] [c=<bytes>]" (element sizes of the tall operand and of the
            # result as stored; 4 where not stated)
            p = tag.split()
            m_, n_, k_ = (float(x) for x in p[2].split("x"))
            ea = next((float(w[2:]) for w in p if w.startswith("a=")), 4.0)
            ec = next((float(w[2:]) for w in p if w.startswith("c=")), 4.0)
            em = next((float(w[2:]) for w in p if w.startswith("m=")), 4.0) if "mask" in p else 0.0   # a mask read along with C
            gq["bytes"] += calls * (ea * m_ * k_ + (ec + em) * m_ * n_ + 4.0 * k_ * n_)
        elif name == "gemm_tn_stream_kernel":
            # both tall operands streamed once (tag: "TN stream MxNxK bf16 a=<bytes> b=<bytes>"); the result is small
            p = tag.split()
            m_, n_, k_ = (float(x) for x in p[2].split("x"))
            ea = next((float(w[2:]) for w in p if w.startswith("a=")), 2.0)
            eb = next((float(w[2:]) for w in p if w.startswith("b=")), 2.0)
            gq["bytes"] += calls * k_ * (ea * m_ + eb * n_)
            gq["flops"] += calls * 2.0 * m_ * n_ * k_
        elif name == "spmm_main_kernel":
            d = int(tag.split("d=")[1].split()[0])
            w = tag.split()
            ein = next((float(x[3:]) for x in w if x.startswith("in=")), 2.0 if "bf16 in" in tag else 4.0)
            eout = next((float(x[4:]) for x in w if x.startswith("out=")), 4.0)
            edo = next((float(x[3:]) for x in w if x.startswith("dO=")), 0.0)      # the loss epilogue also writes the gradient rows
            # compulsory traffic: CSR once, every input row once, the output once
            gq["bytes"] += calls * (8.0 * nnz_avg + 4.0 * (cfg.B + 1) + cfg.B * d * (ein + eout + edo))
    total_ms = sum(v["ms"] for v in groups.values())
    dom_name, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
    sp = [v for k, v in groups.items() if k.startswith("spmm_main_kernel")]
    sparse_ms, sparse_bytes = sum(v["ms"] for v in sp), sum(v["bytes"] for v in sp)
    if args.breakdown:
        for name, tag, calls, ms in recs:
            print("  %-28s %-44s calls %3d  avg us %9.2f" % (name, tag, calls, 1e3 * ms / calls), file=sys.stderr)
        for k, v in sorted(groups.items(), key=lambda kv: -kv[1]["ms"]):
            print("%-44s calls/step %5.1f  us/step %9.2f  avg us %8.2f" %
                  (k, v["calls"] / nprof, 1e3 * v["ms"] / nprof, 1e3 * v["ms"] / v["calls"]), file=sys.stderr)
        print("sum of kernel time per step: %.1f us; wall per step: %.1f us" % (1e3 * total_ms / nprof, 1e6 / steps_per_s),
              file=sys.stderr)
    if dom["flops"] > 0:
        dt = "bf16" if "bf16" in dom_name else "f32"
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
    roofline["algorithmic_per_launch"] = (dom["flops"] or dom["bytes"]) / dom["calls"]
    roofline["share_of_kernel_time"] = dom["ms"] / total_ms if total_ms > 0 else None
    # the sparse products as a whole (all widths), the other large group
    roofline["spmm_all_widths"] = {"bound": "hbm", "achieved": sparse_bytes / (sparse_ms * 1e-3) / 1e9 if sparse_ms > 0 else 0.0,
                                   "peak": PEAK_HBM_GBS, "unit": "GB/s", "us_per_step": 1e3 * sparse_ms / nprof}
    top = sorted(groups.items(), key=lambda kv: -kv[1]["ms"])[:6]
    roofline["top_kernels_us_per_step"] = {k: round(1e3 * v["ms"] / nprof, 1) for k, v in top}

    feat = "bf16" if X.dtype == torch.bfloat16 else "f32"
    act = "bf16" if getattr(st, "bf16_activations", False) else "f32"
    out = {
        "value": steps_per_s, "unit": "steps/s", "steps": K, "warmup": W, "ms_per_step": 1e3 * elapsed / K,
        "dtype": "bf16" if cfg.bf16_mfma else "f32",
        "config": {"workload": "%s: R-MAT N=%d, E=%d stored entries, |S|=%d, %s, features stored %s, activations stored %s, "
                               "%d timed mini-batches with sampler counters %s"
                               % (label, cfg.N, g.E, cfg.B,
                                  ("complete model %d-[%d x %d]-%d with dropout 0.1 and Adam"
                                   % (cfg.d_in, cfg.hidden, max(cfg.layers - 1, 1), cfg.classes)) if model
                                  else "GCN " + "-".join(map(str, cfg.dims)), feat, act, K,
                                  ("0..%d" % (K - 1)) if not use_graph or cyc >= K else
                                  ("0..%d repeated (cycle of %d captured steps)" % (cyc - 1, cyc))),
                   "fuse_slice": not args.no_fuse_slice, "fuse_relu_bwd": not args.no_fuse_relu_bwd, "fuse_loss": ("keep-logits" if st.keep_logits else "drop-logits") if getattr(st, "fuse_loss", False) else "off",
                   "side_stream_dw": args.side_dw and not args.no_overlap,
                   "overlap_sampling": not args.no_overlap, "hip_graph": use_graph,
                   "graph_steps": n_graph, "eager_steps": K - n_graph,
                   "warmup_extra_graph_replays": 1 if use_graph else 0,
                   "single_stream_steps_per_s": single_stream_steps_per_s, "avg_induced_entries": nnz_avg,
                   "kernel_time_us_per_step": 1e3 * total_ms / nprof},
        "roofline": roofline,
    }
    return out, st


def cpu_baseline(args, si, torch, cfg, g, X, weights):
    """The oracle on the host cores on a bounded sample of the workload, in steps/s.

    One step is timed stage by stage.  The sampler (a sort of all N keys) and the extraction (a scan of
    the sampled rows) are timed whole.  The layers (forward, loss, backward) are timed whole when a flop
    estimate puts them under ten seconds; otherwise on the mini-batch induced by every r-th vertex of the
    same sample, their time multiplied by r (the dense products, which dominate, are linear in the number
    of rows).  Where a whole step is short, several whole steps with consecutive counters are timed."""
    import numpy as np
    import oracle
    wnp = [(W.double().cpu().numpy(), b.double().cpu().numpy()) for W, b in weights]
    rp, ci = g.rowptr.cpu().numpy(), g.colidx.cpu().numpy()
    log("%s: graph copied to the host for the oracle" % cfg.name)

    def rows_for(S):       # the slice: rows handed over as data, not timed as oracle work
        St = torch.as_tensor(S.astype(np.int64))
        Xs = X[St.to(X.device)].float().cpu().numpy().astype(np.float64)
        ys = si.labels_for(St, cfg.classes, cfg.label_seed).numpy()
        return Xs, ys

    def layers(S):
        rpS, ciS, vS = oracle.induced_csr(cfg.N, rp, ci, S)
        Xs, ys = rows_for(S)
        c0 = time.perf_counter()
        oracle.layers_step(rpS, ciS, vS, Xs, ys, wnp, bf16=cfg.bf16_mfma)
        return time.perf_counter() - c0

    def stages(t):
        c0 = time.perf_counter()
        S = oracle.sample_uniform(cfg.N, cfg.B, cfg.sampler_seed, t)
        c1 = time.perf_counter()
        oracle.induced_csr(cfg.N, rp, ci, S)
        c2 = time.perf_counter()
        return S, c1 - c0, c2 - c1

    dims = cfg.dims
    flops = 6.0 * cfg.B * sum(dims[l] * dims[l + 1] for l in range(cfg.layers))
    r = 1
    while flops / r > 10.0 * 15e9 and r < 1024:      # plain C loops on all cores: about 15 GFLOP/s
        r *= 2
    layers(np.arange(min(cfg.B, 1024), dtype=np.int32))       # warm-up: library load, thread pool
    S, a, b = stages(0)
    lay = layers(S[::r].copy())
    step_s = a + b + lay * r
    log("%s: oracle sampler %.2f s, extraction %.2f s, layers %.2f s at |S|/%d" % (cfg.name, a, b, lay, r))
    cores = oracle.num_threads()
    if r == 1:
        n = int(max(0, min(49, (args.cpu_seconds - step_s) // max(step_s, 1e-3))))
        total = step_s
        for t in range(1, n + 1):
            S, a, b = stages(t)
            total += a + b + layers(S)
        return {"value": (n + 1) / total, "unit": "steps/s", "cores": cores, "kind": "oracle",
                "sample": "%d whole steps (sampler counters 0..%d) of the same workload: sampler, extraction and "
                          "layers (forward, loss, backward), %.1f s of oracle time" % (n + 1, n, total)}
    return {"value": 1.0 / step_s, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": "one step (sampler counter 0), stage by stage: sampler over all N = %d keys (%.1f s) and extraction "
                      "of the whole |S| = %d mini-batch (%.1f s) timed whole; forward + loss + backward of the layers "
                      "timed on the mini-batch induced by every %d-th sampled vertex (%d rows, %.1f s) and multiplied "
                      "by %d" % (cfg.N, a, cfg.B, b, r, len(S[::r]), lay, r)}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the single-GPU hot path; --gpus N with N > 1 is not supported "
              "(no collectives are part of it)", file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2604_02651_amd as sg
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    log("torch and libsgnn loaded")
    dev = "cuda:0"
    graph_req = "off" if args.no_graph else args.graph
    cfg = si.CONFIGS[args.config]
    model = args.workload == "model"
    fdt = torch.bfloat16 if cfg.bf16_features and not model else torch.float32
    g, X, labels, weights = make_inputs(si, torch, cfg, dev, fdt)
    res, st = measure(args, sg, si, torch, cfg, g, X, labels, weights, graph_req, cfg.name)

    def calibrate():
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            sg.sgnn_copy_f32(st.ctx, src, dst)
        torch.cuda.synchronize()

    if args.profile_steps_only:
        if args.calibrate_copy:
            calibrate()
        return
    out = {"metric": METRIC, "value": res["value"], "unit": res["unit"], "n_gpus": 1, "steps": res["steps"],
           "warmup": res["warmup"], "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
           "roofline": res["roofline"]}

    if args.calibrate_copy:
        calibrate()

    del st
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and not model:
        out["cpu_baseline"] = cpu_baseline(args, si, torch, cfg, g, X, weights)
        log("oracle leg done: %.4f steps/s" % out["cpu_baseline"]["value"])

    extras = args.extras
    if extras == "auto":
        extras = "dense,xlarge_f32_features" if (cfg.name == "xlarge" and not model) else "none"
    others = {}
    for name in [e for e in extras.split(",") if e and e != "none"]:
        try:
            if name == "xlarge_f32_features":
                c2 = si.CONFIGS["xlarge"]
                g2 = g if cfg.name == "xlarge" else None
                del X
                X = None
                gc.collect(); torch.cuda.empty_cache()
                g2, X2, l2, w2 = make_inputs(si, torch, c2, dev, torch.float32, graph=g2)
            else:
                c2 = si.CONFIGS[name]
                g2, X2, l2, w2 = make_inputs(si, torch, c2, dev, torch.float32)
            r2, st2 = measure(args, sg, si, torch, c2, g2, X2, l2, w2, graph_req, name)
            others[name] = {"value": r2["value"], "unit": "steps/s", "ms_per_step": r2["ms_per_step"], "dtype": r2["dtype"],
                            "workload": r2["config"]["workload"], "hip_graph": r2["config"]["hip_graph"],
                            "single_stream_steps_per_s": r2["config"]["single_stream_steps_per_s"],
                            "roofline": r2["roofline"]}
            del st2, X2, l2, w2, g2
            gc.collect(); torch.cuda.empty_cache()
        except Exception as e:       # a sub-object must never cost the headline line
            others[name] = {"error": "%s: %s" % (type(e).__name__, e)}
            log("extra workload %s failed: %s" % (name, e))
    if others:
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
