"""Pins for the oracle's Philox generator and uniform sampler (Eq. 20)."""
import os

import numpy as np
import pytest

import oracle
from helpers import philox_py, vertex_key_py

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == out
        assert philox_py(ctr, key) == out


def test_philox_matches_bigint_version_on_random_inputs():
    rng = np.random.default_rng(5)
    for _ in range(200):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64)
        assert list(oracle.philox4x32_10(ctr, key)) == philox_py(ctr, key)


def test_philox_round_count_matters():
    # a 9- or 11-round variant gives different words: the round count is pinned by the vectors
    assert philox_py([0] * 4, [0] * 2, 9) != philox_py([0] * 4, [0] * 2, 10)


def test_vertex_key_layout():
    for seed, step in [(0, 0), (7, 3), (2**40 + 5, 2**33 + 1)]:
        for v in [0, 1, 2, 3, 1000, 1001, 2**31 - 2]:
            assert oracle.vertex_key(seed, step, v) == vertex_key_py(seed, step, v)
    # even/odd neighbours share a block but take different words
    assert oracle.vertex_key(0, 0, 10) != oracle.vertex_key(0, 0, 11)
    keys = oracle.vertex_keys(3, 9, 50)
    assert [int(k) for k in keys] == [vertex_key_py(3, 9, v) for v in range(50)]


def test_seed_and_step_are_not_interchangeable():
    # the paper adds seed and step, which would make (0,1) and (1,0) collide; here they differ
    a = oracle.sample_uniform(1000, 100, 0, 1)
    b = oracle.sample_uniform(1000, 100, 1, 0)
    c = oracle.sample_uniform(1000, 100, 0, 0)
    assert not np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(b, c)


@pytest.mark.parametrize("N,B", [(1, 1), (2, 1), (65, 64), (1000, 1), (1000, 999), (4096, 1024), (12345, 777)])
def test_sample_shape_and_order(N, B):
    S = oracle.sample_uniform(N, B, 0, 0)
    assert S.dtype == np.int32 and S.shape == (B,)
    assert np.all(np.diff(S) > 0)
    assert S[0] >= 0 and S[-1] < N
    assert np.array_equal(S, oracle.sample_uniform(N, B, 0, 0))


def test_sample_all_vertices():
    assert np.array_equal(oracle.sample_uniform(777, 777, 5, 5), np.arange(777, dtype=np.int32))


def test_sample_invalid():
    for N, B in [(10, 0), (10, 11)]:
        with pytest.raises(ValueError):
            oracle.sample_uniform(N, B, 0, 0)


def test_sample_equals_independent_threshold_selection():
    # second derivation: B-th smallest (key, v) as a threshold, then a filter over all vertices
    for (N, B, seed, step) in [(5000, 1234, 0, 0), (4096, 1024, 0, 3), (999, 500, 11, 2)]:
        keys = [vertex_key_py(seed, step, v) for v in range(N)]
        pairs = sorted(zip(keys, range(N)))
        thr = pairs[B - 1]
        sel = np.array([v for v in range(N) if (keys[v], v) <= thr], np.int32)
        assert np.array_equal(sel, oracle.sample_uniform(N, B, seed, step))


def test_sample_nested_in_B():
    # bottom-B sets are nested: the sample of size B is contained in the sample of size B+1
    a = set(oracle.sample_uniform(3000, 100, 2, 4).tolist())
    b = set(oracle.sample_uniform(3000, 101, 2, 4).tolist())
    assert a < b and len(b - a) == 1


def test_inclusion_probabilities():
    # Eq. 20: Pr[v in S] = B/N, Pr[u,v in S] = B(B-1)/(N(N-1))
    N, B, T = 64, 16, 4000
    counts = np.zeros(N)
    pair = 0
    for t in range(T):
        S = oracle.sample_uniform(N, B, 123, t)
        counts[S] += 1
        pair += int(0 in S and 1 in S) + int(10 in S and 53 in S)
    p = B / N
    sigma = np.sqrt(T * p * (1 - p))
    assert np.all(np.abs(counts - T * p) < 5 * sigma)
    # chi-square of the per-vertex counts stays in a wide band around its mean
    chi2 = ((counts - T * p) ** 2 / (T * p * (1 - p))).sum()
    assert 20 < chi2 < 130
    pp = B * (B - 1) / (N * (N - 1))
    assert abs(pair - 2 * T * pp) < 5 * np.sqrt(2 * T * pp * (1 - pp))


def test_subset_uniformity_small():
    # N=5, B=2: the 10 subsets are equally likely
    from collections import Counter
    T = 5000
    c = Counter(tuple(oracle.sample_uniform(5, 2, 9, t).tolist()) for t in range(T))
    assert len(c) == 10
    for n in c.values():
        assert abs(n - T / 10) < 5 * np.sqrt(T * 0.1 * 0.9)
