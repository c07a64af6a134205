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


# ---------------------------------------------------------------- matrix form of the sample (Eq. 7 under Sec. 3.1)

def test_matrix_sample_is_a_product_of_row_and_column_strata():
    rows, cols, s = 300, 1000, 0.01
    r, c = oracle.sample_matrix_shape(rows, cols, s)
    target = oracle.sample_count(rows * cols, s)
    assert r == round(rows * math.sqrt(s)) == 30 and c == math.ceil(target / r) == 100
    assert r * c >= target and r * (c - 1) < target                    # the least column count that reaches ceil(s d)
    idx, shape = oracle.sample_indices_block(rows * cols, rows, cols, s, seed=3, block=2)
    assert shape == (r, c) and idx.size == r * c and np.all(np.diff(idx.astype(np.int64)) > 0)
    ri, ci = (idx // np.uint64(cols)).reshape(r, c), (idx % np.uint64(cols)).reshape(r, c)
    assert np.all(ri == ri[:, :1]) and np.all(ci == ci[:1, :])         # a Cartesian product
    rsel, csel = ri[:, 0].astype(np.int64), ci[0, :].astype(np.int64)
    assert np.all(rsel >= np.arange(r) * rows // r) and np.all(rsel < (np.arange(r) + 1) * rows // r)     # one row per stratum
    assert np.all(csel >= np.arange(c) * cols // c) and np.all(csel < (np.arange(c) + 1) * cols // c)
    again, _ = oracle.sample_indices_block(rows * cols, rows, cols, s, seed=3, block=2)
    other, _ = oracle.sample_indices_block(rows * cols, rows, cols, s, seed=4, block=2)
    assert np.array_equal(idx, again) and not np.array_equal(idx, other)


def test_matrix_sample_shapes_at_the_edges():
    assert oracle.sample_matrix_shape(64, 64, 1.0) == (64, 64)
    idx, shape = oracle.sample_indices_block(64 * 48, 64, 48, 1.0, 1, 0)
    assert shape == (64, 48) and np.array_equal(idx, np.arange(64 * 48, dtype=np.uint64))   # s = 1: the block itself
    assert oracle.sample_matrix_shape(64, 64, 0.001) == (2, 3)          # 64 sqrt(0.001) = 2.02 rows, ceil(5 / 2) columns
    assert oracle.sample_matrix_shape(20, 20, 0.001) is None            # one row: too thin for a matrix form
    assert oracle.sample_matrix_shape(1, 5000, 0.5) is None and oracle.sample_matrix_shape(5000, 1, 0.5) is None
    idx, shape = oracle.sample_indices_block(400, 20, 20, 0.001, 1, 0)
    assert shape == (0, 0) and idx.size == 1                             # falls back to the flat draw
    for rows, cols, s in ((4096, 4096, 0.001), (4096, 11008, 0.001), (32000, 4096, 0.01), (2, 300001, 0.1), (257, 255, 0.37)):
        got = oracle.sample_matrix_shape(rows, cols, s)
        target = oracle.sample_count(rows * cols, s)
        if got:
            r, c = got
            assert 2 <= r <= rows and 2 <= c <= cols and (r * c >= target or c == cols) and r * c < target + r


def test_matrix_sample_rows_and_columns_are_included_uniformly():
    rows, cols, s = 40, 50, 0.04                              # 8 row strata of 5, 10 column strata of 5
    r, c = oracle.sample_matrix_shape(rows, cols, s)
    assert (r, c) == (8, 10)
    hits = np.zeros((rows, cols))
    n_seeds = 3000
    for seed in range(n_seeds):
        idx, _ = oracle.sample_indices_block(rows * cols, rows, cols, s, seed, 0)
        hits.reshape(-1)[idx.astype(np.int64)] += 1
    p = hits / n_seeds
    want = (r / rows) * (c / cols)
    assert p.mean() == pytest.approx(want, rel=1e-12)
    assert np.all(np.abs(p - want) < 6 * math.sqrt(want * (1 - want) / n_seeds))


def test_structure_residual_of_the_sampled_sub_matrix():
    """A rank-one second moment stays rank one on any sub-matrix (F = 0 dense and sampled); for a matrix with
    structure the sampled F approaches the dense one as the ratio grows."""
    rows, cols = 200, 300
    a, b = np.exp(RNG.standard_normal(rows)), np.exp(RNG.standard_normal(cols))
    gs_rank1 = [np.outer(np.sqrt(a), np.sqrt(b)).astype(np.float32).reshape(-1)] * 3       # v ~ a b^T
    noise = np.exp(0.3 * RNG.standard_normal((rows, cols)))
    gs_full = [(np.outer(np.sqrt(a), np.sqrt(b)) * noise * RNG.standard_normal((rows, cols))).astype(np.float32).reshape(-1) for _ in range(6)]
    for gs, dense_is_zero in ((gs_rank1, True), (gs_full, False)):
        dense = oracle.Block(rows * cols)
        for g in gs:
            dense.step(g)
        F_dense = dense.structure_residual(rows, cols)
        for s, tol in ((0.04, 0.2), (0.25, 0.1), (0.6, 0.04)):      # a small sub-matrix is fitted better by rank one: F is biased low
            idx, (r, c) = oracle.sample_indices_block(rows * cols, rows, cols, s, 11, 0)
            blk = oracle.Block(idx.size)
            for g in gs:
                blk.step(g[idx.astype(np.int64)])
            F = blk.structure_residual(r, c)
            if dense_is_zero:
                assert F_dense < 1e-6 and F < 1e-6
            else:
                assert F_dense > 0.3 and F == pytest.approx(F_dense, abs=tol)
