"""Block partitioner (App. C.2, Algorithm 2): the Python oracle pinned by hand-worked cases and
invariants; the library's baoc_partition bit-exact against the oracle."""
import ctypes as C
import itertools

import numpy as np
import pytest

import paper_2605_04711_amd as B
from oracle.partition import partition as oracle_partition
from paper_2605_04711_amd import binding

RNG = np.random.default_rng(21)


def lib_partition(numel, z, weights=None, alpha=0.01):
    return binding.partition(numel, z, weights, alpha)


def test_identical_statistics_collapse_to_one_block():
    ids, n, tau = oracle_partition([100] * 6, [[0.3, 0.7]] * 6, alpha=0.05)
    assert ids == [0] * 6 and n == 1 and tau == 0.0


def test_two_plateaus_split_at_the_step():
    # five large units at z = 0, five at z = 1: pairwise Delta is 0 (20 pairs) or 1 (25 pairs),
    # so the upper quartile is 1 and nothing *exceeds* it: one block.
    z = [[0.0]] * 5 + [[1.0]] * 5
    ids, n, tau = oracle_partition([1000] * 10, z, alpha=0.01)
    assert tau == 1.0 and n == 1
    # three plateaus 0, 0.5, 1 of 6, 2, 2 units: 17 pairs at 0, 16 at 0.5, 12 at 1; position 0.75 * 44 = 33
    # lands on the first 1 -> tau = 1, still one block
    z = [[0.0]] * 6 + [[0.5]] * 2 + [[1.0]] * 2
    ids, n, tau = oracle_partition([1000] * 10, z, alpha=0.01)
    deltas = sorted(abs(a[0] - b[0]) for a, b in itertools.combinations(z, 2))
    assert tau == pytest.approx(float(np.quantile(deltas, 0.75)), abs=1e-15) and tau == 1.0 and n == 1
    # fourteen units at 0 and two at 1: 92 of 120 pairs are 0, position 0.75 * 119 = 89.25 is a 0:
    # tau = 0 and the one step exceeds it
    z = [[0.0]] * 14 + [[1.0]] * 2
    ids, n, tau = oracle_partition([1000] * 16, z, alpha=0.01)
    assert tau == 0.0 and ids == [0] * 14 + [1] * 2 and n == 2


def test_hand_worked_five_units():
    # sizes 50 10 50 50 40 (total 200), alpha = 0.1 -> n_min = 20; z = 0, 0.9, 1, 1, 0.1
    # pairwise Delta: .9 1 1 .1 | .1 .1 .8 | 0 .9 | .9  -> sorted 0 .1 .1 .1 .8 .9 .9 .9 1 1,
    # position 0.75 * 9 = 6.75 -> 0.9 + 0.75 * (0.9 - 0.9) = 0.9
    # filtering: unit 1 (10 < 20) goes to its closer neighbour, unit 2 (Delta .1 vs .9)
    #   -> temporary blocks [0] [1 2] [3] [4]; stats 0, (9+50)/60 = .98333, 1, .1
    # formation: Delta([0],[1 2]) = .98333 > .9 keep; Delta([1 2],[3]) = .01667 merge; Delta([3],[4]) = .9 not > .9 merge
    #   -> [0] | [1 2] [3] [4]
    # split of the second block: cut after [1 2]: .98333 vs (50+4)/90 = .6 -> .38333; cut after [3]: 109/110 = .99091 vs .1 -> .89091
    #   best .89091 is not > .9 -> no split.  Result: 2 blocks.
    ids, n, tau = oracle_partition([50, 10, 50, 50, 40], [[0.0], [0.9], [1.0], [1.0], [0.1]], alpha=0.1)
    assert tau == pytest.approx(0.9, abs=1e-15) and ids == [0, 1, 1, 1, 1] and n == 2


def test_smooth_ramp_stays_one_block():
    # z = 0, 1/8, ..., 1 on nine equal units: Delta = k/8 for 9-k pairs; position 0.75 * 35 = 26.25 falls
    # among the five pairs at 5/8 -> tau = 0.625.  Adjacent steps are 1/8: one formed block.  Any cut
    # separates means (p-1)/16 and (p+8)/16, difference 9/16 < tau: no split.
    ids, n, tau = oracle_partition([100] * 9, [[k / 8.0] for k in range(9)], alpha=0.05)
    assert tau == 0.625 and n == 1 and ids == [0] * 9


def test_small_unit_joins_the_statistically_closest_neighbour():
    ids, n, _ = oracle_partition([1000, 5, 1000, 1000, 1000, 1000], [[0.0], [0.95], [1.0], [0.0], [1.0], [0.0]], alpha=0.01)
    assert ids[1] == ids[2]
    ids, n, _ = oracle_partition([1000, 5, 1000, 1000, 1000, 1000], [[0.0], [0.05], [1.0], [0.0], [1.0], [0.0]], alpha=0.01)
    assert ids[1] == ids[0]


def test_weights_select_the_component_that_matters():
    z = [[0.0, float(j % 2)] for j in range(14)] + [[1.0, 0.5]] * 2
    a = oracle_partition([100] * 16, z, weights=[1.0, 0.0], alpha=0.01)       # only the step in component 0 counts
    assert a[0] == [0] * 14 + [1] * 2 and a[2] == 0.0
    b = oracle_partition([100] * 16, z, weights=[0.0, 1.0], alpha=0.01)       # alternating component: tau = 1, no cut
    assert b[1] == 1 and b[2] == 1.0


def invariants(numel, ids, n, alpha):
    assert ids[0] == 0 and all(0 <= b - a <= 1 for a, b in zip(ids, ids[1:])) and ids[-1] == n - 1
    sizes = [sum(numel[j] for j in range(len(ids)) if ids[j] == b) for b in range(n)]
    if n > 1:
        assert min(sizes) >= alpha * sum(numel)


@pytest.mark.parametrize("trial", range(40))
def test_library_matches_oracle_and_invariants_hold(trial):
    m = int(RNG.integers(1, 40)); K = int(RNG.integers(1, 6))
    numel = [int(x) for x in RNG.integers(1, 5000, m)]
    kind = trial % 3
    if kind == 0:
        z = RNG.random((m, K))
    elif kind == 1:                                   # plateaus with noise
        z = np.repeat(RNG.random((max(1, m // 5) + 1, K)), 5, axis=0)[:m] + 0.02 * RNG.random((m, K))
    else:                                             # many exact ties
        z = RNG.integers(0, 3, (m, K)) / 2.0
    w = None if trial % 4 else RNG.random(K)
    alpha = [0.0, 0.01, 0.05, 0.2][trial % 4]
    want = oracle_partition(numel, z.tolist(), None if w is None else w.tolist(), alpha)
    got = lib_partition(numel, z, w, alpha)
    assert list(got[0]) == want[0] and got[1] == want[1] and got[2] == want[2]
    invariants(numel, want[0], want[1], alpha)


def test_library_rejects_bad_arguments():
    lib = B.load_library()
    assert lib.baoc_partition(None, None, 0, 0, None, 0.1, None, None, None) == binding.ERR_INVALID
    with pytest.raises(B.BaocError):
        lib_partition([1, 2], np.zeros((2, 1)), None, -0.5)
    with pytest.raises(B.BaocError):
        lib_partition([1, 0], np.zeros((2, 1)), None, 0.1)
    with pytest.raises(B.BaocError):
        lib_partition([1, 2], np.array([[0.0], [np.nan]]), None, 0.1)
    with pytest.raises(B.BaocError) as e:                              # tau is a quantile over all unit pairs
        lib_partition(np.ones(40000, np.uint64), np.zeros((40000, 1)), None, 0.0)
    assert e.value.status == binding.ERR_UNSUPPORTED
