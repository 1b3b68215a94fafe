"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

Nothing here is part of the method: this module only makes graphs, features, labels and
weights.  All integer-valued outputs (graph structure, labels) are a pure function of the
seed, built from a 64-bit integer mixing function evaluated with torch integer ops, so
they are bit-identical on the CPU and on the GPU.  Floating-point outputs (features,
weights) are made on the requested device and are handed to both sides as data.

The graphs stand in for the public datasets the paper trains on (co-purchase, social and
citation graphs, Section VI "Datasets"): they are R-MAT graphs with the vertex count, edge
count and feature width of those datasets, not the datasets themselves.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

_M64 = (1 << 64) - 1


def _i64(x: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant as a Python int in int64 range."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _i64(0xBF58476D1CE4E5B9)
_C2 = _i64(0x94D049BB133111EB)
_GOLD = 0x9E3779B97F4A7C15


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def mix64(idx: torch.Tensor, seed: int) -> torch.Tensor:
    """Bijective 64-bit mixer (xor-shift / multiply finaliser) of idx, offset by the seed.

    idx is an int64 tensor; the result is an int64 tensor holding the 64 mixed bits.
    """
    off = _i64((seed + 1) * _GOLD)
    z = idx + off
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    z = z ^ _lsr(z, 31)
    return z


def uniform_bits(idx: torch.Tensor, seed: int, bits: int) -> torch.Tensor:
    """Top `bits` (<= 53) of the mixed value as a non-negative int64."""
    return _lsr(mix64(idx, seed), 64 - bits)


def uniform01(idx: torch.Tensor, seed: int) -> torch.Tensor:
    """Uniform in (0, 1) as float64, 53 bits."""
    return (uniform_bits(idx, seed, 53).to(torch.float64) + 0.5) * (1.0 / (1 << 53))


# ----------------------------------------------------------------------------------------------
# R-MAT graph
# ----------------------------------------------------------------------------------------------

def _rmat_edges(e0: int, count: int, scale: int, seed: int, abcd, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Endpoints of R-MAT draws number e0 .. e0+count-1 (one quadrant choice per bit level)."""
    a, b, c, _ = abcd
    t1 = int(round(a * (1 << 24)))
    t2 = int(round((a + b) * (1 << 24)))
    t3 = int(round((a + b + c) * (1 << 24)))
    e = torch.arange(e0, e0 + count, dtype=torch.int64, device=device)
    u = torch.zeros(count, dtype=torch.int64, device=device)
    v = torch.zeros(count, dtype=torch.int64, device=device)
    for level in range(scale):
        r = uniform_bits(e * scale + level, seed, 24)
        row_bit = (r >= t2).to(torch.int64)                      # quadrants c, d
        col_bit = (((r >= t1) & (r < t2)) | (r >= t3)).to(torch.int64)  # quadrants b, d
        u = (u << 1) | row_bit
        v = (v << 1) | col_bit
    return u, v


@dataclass
class Graph:
    """Canonical CSR of A + I: sorted unique columns, exactly one self-loop per row."""
    N: int
    rowptr: torch.Tensor   # int64 [N+1]
    colidx: torch.Tensor   # int32 [E]

    @property
    def E(self) -> int:
        return int(self.colidx.numel())


def rmat_graph(N: int, undirected_edges: int, seed: int = 1234, device="cpu",
               abcd=(0.57, 0.19, 0.19, 0.05), permute: bool = True,
               chunk: int = 1 << 25, max_rounds: int = 400) -> Graph:
    """R-MAT graph on N vertices with exactly `undirected_edges` distinct undirected edges
    (no self edges among them), symmetrised, plus one self-loop per vertex.

    Draws with an endpoint >= N or with equal endpoints are rejected, duplicates are merged, and
    draws continue until the target count of distinct edges is reached; the surplus of the last
    round is trimmed by a seeded pseudo-random order.  Vertex ids are then relabelled by a seeded
    bijection so that degree is not correlated with id.
    """
    device = torch.device(device)
    max_pairs = N * (N - 1) // 2
    if undirected_edges > max_pairs:
        raise ValueError("more edges requested than vertex pairs exist")
    scale = max(1, math.ceil(math.log2(max(N, 2))))
    keys = torch.empty(0, dtype=torch.int64, device=device)
    drawn = 0
    for _ in range(max_rounds):
        need = undirected_edges - int(keys.numel())
        if need <= 0:
            break
        count = int(min(chunk, max(1024, need * 2)))
        u, v = _rmat_edges(drawn, count, scale, seed, abcd, device)
        drawn += count
        ok = (u < N) & (v < N) & (u != v)
        u, v = u[ok], v[ok]
        lo, hi = torch.minimum(u, v), torch.maximum(u, v)
        keys = torch.unique(torch.cat([keys, lo * N + hi]))
    if int(keys.numel()) < undirected_edges:
        raise RuntimeError("R-MAT generator did not reach the requested edge count")
    if int(keys.numel()) > undirected_edges:
        order = torch.argsort(mix64(keys, seed + 7919))
        keys = keys[order[:undirected_edges]]
    lo, hi = keys // N, keys % N
    del keys
    if permute:
        perm = torch.argsort(mix64(torch.arange(N, dtype=torch.int64, device=device), seed + 104729))
        lo, hi = perm[lo], perm[hi]
    loops = torch.arange(N, dtype=torch.int64, device=device)
    src = torch.cat([lo, hi, loops])
    dst = torch.cat([hi, lo, loops])
    del lo, hi, loops
    dkeys, _ = torch.sort(src * N + dst)
    del src, dst
    rows = dkeys // N
    colidx = (dkeys % N).to(torch.int32)
    del dkeys
    counts = torch.bincount(rows, minlength=N)
    rowptr = torch.zeros(N + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(counts, 0)
    return Graph(N=N, rowptr=rowptr, colidx=colidx)


def rmat_graph_bucketed(N: int, undirected_edges: int, seed: int = 1234, device="cpu",
                        abcd=(0.57, 0.19, 0.19, 0.05), permute: bool = True, chunk: int = 1 << 27,
                        buckets: int = 64, oversample: float = 1.0) -> Graph:
    """R-MAT graph for sizes at which one global sort of all directed edges is impractical
    (billions of entries).  Same generator and rejection rules as rmat_graph, but the number of
    DRAWS is fixed (undirected_edges * oversample accepted draws) instead of the number of distinct
    edges, so the distinct count comes out slightly below the target (duplicates are merged); the
    actual count is Graph.E.  Directed keys are sorted per chunk, split into `buckets` row ranges,
    and every bucket is merged and deduplicated on its own.
    """
    device = torch.device(device)
    scale = max(1, math.ceil(math.log2(max(N, 2))))
    want = int(undirected_edges * oversample)
    perm = None
    if permute:
        perm = torch.argsort(mix64(torch.arange(N, dtype=torch.int64, device=device), seed + 104729))
    rows_per_bucket = (N + buckets - 1) // buckets
    bounds = torch.arange(0, buckets + 1, dtype=torch.int64, device=device) * rows_per_bucket * N
    parts = [[] for _ in range(buckets)]
    accepted, drawn = 0, 0
    while accepted < want:
        u, v = _rmat_edges(drawn, chunk, scale, seed, abcd, device)
        drawn += chunk
        ok = (u < N) & (v < N) & (u != v)
        u, v = u[ok], v[ok]
        del ok
        if accepted + int(u.numel()) > want:
            keep = want - accepted
            u, v = u[:keep], v[:keep]
        accepted += int(u.numel())
        if perm is not None:
            u, v = perm[u], perm[v]
        keys = torch.cat([u * N + v, v * N + u])
        del u, v
        keys, _ = torch.sort(keys)
        cut = torch.searchsorted(keys, bounds).tolist()
        for b in range(buckets):
            if cut[b + 1] > cut[b]:
                parts[b].append(keys[cut[b]:cut[b + 1]].clone())
        del keys
    del perm
    counts = torch.zeros(N, dtype=torch.int64, device=device)
    cols = []
    for b in range(buckets):
        r0, r1 = b * rows_per_bucket, min(N, (b + 1) * rows_per_bucket)
        if r0 >= r1:
            continue
        loops = torch.arange(r0, r1, dtype=torch.int64, device=device)
        k = torch.unique(torch.cat(parts[b] + [loops * N + loops]))
        parts[b] = None
        rows = k // N
        cols.append((k - rows * N).to(torch.int32))
        counts[r0:r1] = torch.bincount(rows - r0, minlength=r1 - r0)
        del k, rows, loops
    colidx = torch.cat(cols)
    del cols
    rowptr = torch.zeros(N + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(counts, 0)
    return Graph(N=N, rowptr=rowptr, colidx=colidx)


def config_graph(cfg: "Config", device="cpu") -> Graph:
    """The graph of a workload configuration (the largest one through the bucketed generator)."""
    if cfg.undirected_edges > (1 << 28):
        # 1.0149 accepted draws per target edge: about 1.5 % of the draws repeat an earlier edge
        return rmat_graph_bucketed(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=device, oversample=1.0149)
    return rmat_graph(cfg.N, cfg.undirected_edges, cfg.graph_seed, device=device)


def graph_from_edges(N: int, edges: List[Tuple[int, int]], device="cpu") -> Graph:
    """Canonical CSR of A + I from an explicit undirected edge list (for hand-made test graphs)."""
    pairs = set()
    for u, v in edges:
        if u != v:
            pairs.add((u, v))
            pairs.add((v, u))
    for v in range(N):
        pairs.add((v, v))
    pairs = sorted(pairs)
    rows = torch.tensor([p[0] for p in pairs], dtype=torch.int64)
    cols = torch.tensor([p[1] for p in pairs], dtype=torch.int32)
    rowptr = torch.zeros(N + 1, dtype=torch.int64)
    rowptr[1:] = torch.cumsum(torch.bincount(rows, minlength=N), 0)
    return Graph(N=N, rowptr=rowptr.to(device), colidx=cols.to(device))


# ----------------------------------------------------------------------------------------------
# features, labels, weights
# ----------------------------------------------------------------------------------------------

def normal_rows(rows: torch.Tensor, d: int, seed: int = 1, dtype=torch.float32) -> torch.Tensor:
    """Standard-normal feature rows for the given vertex ids: entry (v, j) depends only on
    (seed, v, j), so any subset of rows can be regenerated without the whole matrix."""
    rows = rows.to(torch.int64)
    j = torch.arange(d, dtype=torch.int64, device=rows.device)
    idx = (rows[:, None] * d + j[None, :]) * 2
    u1 = uniform01(idx, seed)
    u2 = uniform01(idx + 1, seed)
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
    return z.to(dtype)


def normal_features(N: int, d: int, seed: int = 1, device="cpu", dtype=torch.float32,
                    block: int = 1 << 20) -> torch.Tensor:
    """N x d matrix of N(0,1) draws, row-major."""
    out = torch.empty((N, d), dtype=dtype, device=device)
    for r0 in range(0, N, block):
        r1 = min(N, r0 + block)
        out[r0:r1] = normal_rows(torch.arange(r0, r1, dtype=torch.int64, device=device), d, seed, dtype)
    return out


def uniform_labels(N: int, classes: int, seed: int = 2, device="cpu") -> torch.Tensor:
    idx = torch.arange(N, dtype=torch.int64, device=device)
    return (uniform_bits(idx, seed, 31) % classes).to(torch.int32)


def labels_for(rows: torch.Tensor, classes: int, seed: int = 2) -> torch.Tensor:
    """Labels of the given vertex ids (the same values as uniform_labels(N, ...)[rows])."""
    return (uniform_bits(rows.to(torch.int64), seed, 31) % classes).to(torch.int32)


def glorot_uniform(fan_in: int, fan_out: int, seed: int = 3, device="cpu") -> torch.Tensor:
    """fan_in x fan_out fp32 matrix, U(-l, l) with l = sqrt(6 / (fan_in + fan_out))."""
    lim = math.sqrt(6.0 / (fan_in + fan_out))
    idx = torch.arange(fan_in * fan_out, dtype=torch.int64, device=device)
    w = (uniform01(idx, seed) * 2.0 - 1.0) * lim
    return w.reshape(fan_in, fan_out).to(torch.float32)


def uniform_matrix(rows: int, cols: int, seed: int, device="cpu", lo=-1.0, hi=1.0) -> torch.Tensor:
    idx = torch.arange(rows * cols, dtype=torch.int64, device=device)
    return (uniform01(idx, seed) * (hi - lo) + lo).reshape(rows, cols).to(torch.float32)


# ----------------------------------------------------------------------------------------------
# the five workload configurations
# ----------------------------------------------------------------------------------------------

@dataclass
class Config:
    name: str
    N: int
    undirected_edges: int
    d_in: int
    hidden: int
    layers: int
    classes: int
    B: int
    bf16_mfma: bool = False
    bf16_features: bool = False      # the input features are stored as bfloat16
    steps: int = 1
    graph_seed: int = 1234
    feature_seed: int = 1
    label_seed: int = 2
    weight_seed: int = 3
    sampler_seed: int = 0

    @property
    def dims(self) -> List[int]:
        return [self.d_in] + [self.hidden] * (self.layers - 1) + [self.classes]


CONFIGS = {
    "tiny": Config("tiny", 4096, 32768, 32, 64, 2, 8, 1024),
    "medium": Config("medium", 262144, 2097152, 128, 256, 3, 32, 32768, steps=16),
    "large": Config("large", 2449029, 61859140, 100, 256, 3, 47, 262144, bf16_mfma=True),
    "dense": Config("dense", 232965, 57307946, 602, 256, 2, 41, 65536),
    "xlarge": Config("xlarge", 111059956, 1615685872, 128, 256, 3, 172, 1048576, bf16_mfma=True, bf16_features=True),
}


def layer_weights(cfg: Config, device="cpu") -> List[Tuple[torch.Tensor, torch.Tensor]]:
    """[(W_l, b_l)] for the stack d_in -> hidden -> ... -> classes; biases are small non-zero
    values so that a dropped bias term shows up in parity checks."""
    out = []
    dims = cfg.dims
    for l in range(cfg.layers):
        W = glorot_uniform(dims[l], dims[l + 1], cfg.weight_seed + 10 * l, device)
        b = uniform_matrix(1, dims[l + 1], cfg.weight_seed + 10 * l + 5, device, -0.1, 0.1).reshape(-1)
        out.append((W, b))
    return out
