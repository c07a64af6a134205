"""Pins of the oracle's sparse coordinate sampling (Sec. 3.1)."""
import math

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(5)


def test_sample_size_is_the_ceiling_of_s_d():
    assert oracle.sample_count(4096, 0.001) == 5          # ceil(4.096)
    assert oracle.sample_count(1000, 0.1) == 100
    assert oracle.sample_count(1000, 0.1001) == 101
    assert oracle.sample_count(64, 0.001) == 1            # never empty
    assert oracle.sample_count(7, 1.0) == 7 and oracle.sample_count(7, 5.0) == 7
    for d in (1, 2, 999, 12345, 16_777_216):
        for s in (0.001, 0.01, 0.02, 0.05, 0.1):
            assert oracle.sample_count(d, s) == max(1, min(d, math.ceil(s * d)))


def test_indices_are_a_fixed_ascending_subset_one_per_stratum():
    d, s = 100_003, 0.01
    a = oracle.sample_indices(d, s, seed=3, block=7)
    k = a.size
    assert k == 1001 and np.all(np.diff(a.astype(np.int64)) > 0) and a[-1] < d
    lo = (np.arange(k, dtype=object) * d // k).astype(np.uint64)
    hi = ((np.arange(k, dtype=object) + 1) * d // k).astype(np.uint64)
    assert np.all(a >= lo) and np.all(a < hi)
    assert np.array_equal(a, oracle.sample_indices(d, s, seed=3, block=7))            # fixed after one draw
    assert not np.array_equal(a, oracle.sample_indices(d, s, seed=4, block=7))
    assert not np.array_equal(a, oracle.sample_indices(d, s, seed=3, block=8))


def test_full_ratio_is_every_coordinate_and_reduces_to_dense_profiling():
    d = 777
    idx = oracle.sample_indices(d, 1.0, seed=1, block=0)
    assert np.array_equal(idx, np.arange(d, dtype=np.uint64))
    gs = [RNG.standard_normal(d).astype(np.float32) for _ in range(4)]
    dense, sampled = oracle.Block(d), oracle.Block(idx.size)
    for g in gs:
        dense.step(g); sampled.step(g[idx.astype(np.int64)])
    assert dense.finalize().asdict() == sampled.finalize().asdict()


def test_inclusion_is_uniform():
    d, s = 1000, 0.05
    hits = np.zeros(d)
    n_seeds = 4000
    for seed in range(n_seeds):
        hits[oracle.sample_indices(d, s, seed, 0).astype(np.int64)] += 1
    p = hits / n_seeds
    assert p.mean() == pytest.approx(s, rel=1e-12)
    assert np.all(np.abs(p - s) < 5 * math.sqrt(s * (1 - s) / n_seeds))


def test_sampled_statistics_approach_dense_ones():
    d = 400_000
    base = RNG.standard_normal(d); kappa = np.exp(0.5 * RNG.standard_normal(d))
    gs = [(kappa * (base + RNG.standard_normal(d))).astype(np.float32) for _ in range(6)]
    dense = oracle.Block(d)
    for g in gs:
        dense.step(g)
    D = dense.finalize()
    for s, tol in ((0.01, 0.06), (0.1, 0.02)):
        idx = oracle.sample_indices(d, s, 9, 0).astype(np.int64)
        b = oracle.Block(idx.size)
        for g in gs:
            b.step(g[idx])
        S = b.finalize()
        assert S.rho_bar == pytest.approx(D.rho_bar, abs=tol)
        assert S.A == pytest.approx(D.A, abs=3 * tol)
        assert S.snr == pytest.approx(D.snr, rel=3 * tol)
