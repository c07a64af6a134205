"""Pins of the oracle's normalisation, risk table and allocation solvers."""
import itertools
import math

import numpy as np
import pytest
from scipy.optimize import Bounds, LinearConstraint, milp

import oracle

RNG = np.random.default_rng(7)


# ---------------------------------------------------------------- Eq. 1 and Eq. 11 / App. A

def test_agg_table(golden):
    for name, ya, ym, yd, yf, bits, val in golden("agg_values.txt"):
        assert oracle.agg((int(ya), int(ym), int(yd), int(yf), int(bits))) == float(val), name


def _stats(**kw):
    st = oracle.Stats()
    for k, v in kw.items():
        setattr(st, k, v)
    return st


def test_phi_is_the_linear_risk_plus_regulariser():
    st = _stats(s_A=0.3, s_M=0.5, C_tilde=0.2, s_F=0.1, lQ32=0.0, lQ16=0.01, lQ8=0.7)
    rp = oracle.default_risk_params()
    # worked by hand from Eq. 11 and Eq. 1, gamma = 0.1
    cases = {
        (1, 1, 1, 0, 32): 0.0 + 0.1 * 0,
        (1, 1, 1, 0, 16): 0.01 + 0.1 * 1,
        (1, 1, 1, 0, 8): 0.7 + 0.1 * 3,
        (1, 1, 0, 0, 32): 0.2 + 0.1 * 1,
        (0, 0, 0, 0, 32): 0.3 + 0.5 + 0.2 + 0.1 * 3,
        (0, 1, 0, 0, 16): 0.3 + 0.2 + 0.01 + 0.1 * 3,
        (1, 0, 0, 1, 32): 0.5 + 0.2 + 0.1 + 0.1 * 3,
        (1, 0, 1, 1, 8): 0.5 + 0.1 + 0.7 + 0.1 * 5,
    }
    for cfg, want in cases.items():
        assert oracle.phi(st, cfg, False, rp) == pytest.approx(want, rel=1e-14), cfg
    rp2 = oracle.default_risk_params(gamma=0.5, lambda_pref=0.25)
    assert oracle.phi(st, (1, 1, 1, 0, 8), True, rp2) == pytest.approx(0.7 - 0.25 + 0.5 * 3, rel=1e-14)
    assert oracle.phi(st, (1, 1, 1, 0, 8), False, rp2) == pytest.approx(0.7 + 0.5 * 3, rel=1e-14)


def test_normalisation_anchors():
    # snr: T = 1, beta_m = 0.99 -> rho_snr = (1-beta_m)^2 / (1-beta_v) for any gradient
    g = RNG.standard_normal(999).astype(np.float32)
    b = oracle.Block(999, beta_m=0.99); b.step(g)
    st = b.finalize()
    bm, bv = float(np.float32(0.99)), float(np.float32(0.999))
    snr = (1 - bm) ** 2 / (1 - bv)
    assert st.snr == pytest.approx(snr, rel=1e-5)
    assert st.s_snr == pytest.approx(math.log1p(snr) / 2.0, rel=1e-5)
    assert st.s_rho == 0.0 and st.s_M == 0.0
    # gate off: s_M = s_rho ; distortion and structure inputs
    b = oracle.Block(64)
    e1 = np.zeros(64, np.float32); e1[0] = 1
    g2 = np.zeros(64, np.float32); g2[0] = 0.5; g2[1] = math.sqrt(0.75)
    b.step(e1); b.step(g2)
    on = b.finalize(oracle.default_risk_params(), C_raw=1.5, F_raw=1.7)
    off = b.finalize(oracle.default_risk_params(use_snr_gate=0), C_raw=0.0, F_raw=0.25)
    assert on.s_M == pytest.approx(on.s_rho * on.s_snr, rel=1e-15) and off.s_M == off.s_rho
    assert on.s_rho == pytest.approx(0.75, abs=1e-6)
    assert on.C_tilde == pytest.approx(math.log(2.5), rel=1e-15) and on.s_F == 1.0
    assert off.C_tilde == 0.0 and off.s_F == 0.25
    moved = b.finalize(oracle.default_risk_params(rho_low=0.4, rho_high=0.9))
    assert moved.s_rho == pytest.approx(0.2, abs=1e-6)


def test_precision_risk_is_minus_log_of_clipped_cosine():
    g = RNG.standard_normal(2048).astype(np.float32)
    b = oracle.Block(2048); b.step(g); b.step(-g)
    st = b.finalize()
    assert st.lQ16 == pytest.approx(-math.log(st.Q16 + 1e-12), rel=1e-12)
    assert st.lQ8 == pytest.approx(-math.log(st.Q8 + 1e-12), rel=1e-12)
    assert 1e-12 <= st.Q8 <= 1.0 and 1e-12 <= st.Q16 <= 1.0


def test_profiler_risk_table_rows():
    blocks = [(0, 500), (512, 300)]
    p = oracle.Profiler(blocks)
    for _ in range(3):
        p.step(RNG.standard_normal(812).astype(np.float32))
    cfgs = [(1, 1, 0, 0, 32), (1, 1, 0, 0, 8), (0, 0, 0, 0, 32)]
    stats, phi = p.finalize(cfgs, pref_mask=[0, 1, 0], rp=oracle.default_risk_params(lambda_pref=0.5))
    assert phi.shape == (2, 3)
    for i, st in enumerate(stats):
        assert phi[i, 0] == pytest.approx(st.C_tilde + st.lQ32 + 0.1 * 1, abs=1e-15)
        assert phi[i, 1] == pytest.approx(st.lQ8 - 0.5 + 0.1 * 4, rel=1e-14)
        assert phi[i, 2] == pytest.approx(st.s_A + st.s_M + st.lQ32 + 0.1 * 3, rel=1e-14)


# ---------------------------------------------------------------- Eq. 2 allocation

def random_instance(N, K, int_risk=False, mem_hi=9, tau_units=4):
    risk = RNG.integers(0, 6, (N, K)).astype(np.float64) if int_risk else RNG.random((N, K)) * 3
    mem = RNG.integers(0, mem_hi, (N, K)).astype(np.int64)
    time = RNG.integers(1, tau_units + 1, (N, K)) * 0.5
    b_mem = int(mem.min(1).sum() + RNG.random() * (mem.max(1).sum() - mem.min(1).sum()))
    b_time = float(time.min(1).sum() + RNG.random() * (time.max(1).sum() - time.min(1).sum()))
    return risk, mem, time, b_mem, b_time


def test_hand_worked_instance():
    # two blocks, two configurations; budget 5 forces exactly one block to the cheap configuration;
    # cheapest risk increase is block 1 (0.2 < 0.7)
    risk = np.array([[0.1, 0.8], [0.3, 0.5]])
    mem = np.array([[4, 1], [4, 1]], np.int64)
    time = np.ones((2, 2))
    rc, x, obj, m, t = oracle.allocate_brute(risk, mem, time, 5, 10.0)
    assert rc == 0 and list(x) == [0, 1] and obj == pytest.approx(0.6) and m == 5 and t == 2.0
    rc, x, *_ = oracle.allocate_brute(risk, mem, time, 8, 10.0)
    assert rc == 0 and list(x) == [0, 0]
    rc, x, *_ = oracle.allocate_brute(risk, mem, time, 1, 10.0)
    assert rc == oracle.ORC_INFEASIBLE
    rc, x, *_ = oracle.allocate_brute(risk, mem, time, 8, 1.5)       # time row: sum of r <= 1.5 < 2
    assert rc == oracle.ORC_INFEASIBLE
    rc, x, *_ = oracle.allocate_brute(risk, mem, time, 8, 10.0, forbidden=np.array([[1, 0], [0, 0]]))
    assert rc == 0 and list(x) == [1, 0]
    risk2 = risk.copy(); risk2[0, 0] = np.nan                         # non-finite risk = excluded pair
    rc, x, *_ = oracle.allocate_brute(risk2, mem, time, 8, 10.0)
    assert rc == 0 and list(x) == [1, 0]


def test_slack_budgets_give_per_block_argmin_lowest_index():
    risk = RNG.integers(0, 3, (7, 4)).astype(np.float64)
    mem = RNG.integers(0, 9, (7, 4)); time = RNG.random((7, 4))
    for solver in (oracle.allocate_brute, oracle.allocate_dp):
        rc, x, *_ = solver(risk, mem, np.round(time * 4) / 4, 10 ** 9, 1e6)
        assert rc == 0 and list(x) == list(np.argmin(risk, axis=1))


def test_ties_resolve_to_lexicographically_smallest():
    risk = np.zeros((3, 3)); mem = np.array([[2, 1, 0]] * 3, np.int64); time = np.ones((3, 3))
    # budget 3: all assignments with total memory <= 3 cost 0; smallest vector is (0, 1, 2)
    for solver in (oracle.allocate_brute, oracle.allocate_dp):
        rc, x, *_ = solver(risk, mem, time, 3, 1e6)
        assert rc == 0 and list(x) == [0, 1, 2]
    # explicit enumeration in Python as a third opinion
    best = min((c for c in itertools.product(range(3), repeat=3) if sum(mem[i, c[i]] for i in range(3)) <= 3))
    assert list(best) == [0, 1, 2]


@pytest.mark.parametrize("trial", range(12))
def test_brute_force_and_dynamic_programme_agree(trial):
    N, K = int(RNG.integers(2, 8)), int(RNG.integers(2, 5))
    risk, mem, time, bm, bt = random_instance(N, K, int_risk=(trial % 2 == 0))
    fb = (RNG.random((N, K)) < 0.1).astype(np.uint8) if trial % 3 == 0 else None
    a = oracle.allocate_brute(risk, mem, time, bm, bt, fb)
    b = oracle.allocate_dp(risk, mem, time, bm, bt, fb)
    assert a[0] == b[0]
    if a[0] == 0:
        assert list(a[1]) == list(b[1]) and a[2:] == b[2:]
        x = a[1]
        assert sum(mem[i, x[i]] for i in range(N)) <= bm
        assert sum(time[i, x[i]] for i in range(N)) <= bt + 1e-9
        if fb is not None:
            assert not any(fb[i, x[i]] for i in range(N))


def solve_with_library_milp(risk, mem, time, bm, bt):
    """Eq. 2 handed to an off-the-shelf MILP solver, as the paper does."""
    N, K = risk.shape
    A_one = np.kron(np.eye(N), np.ones((1, K)))
    cons = [LinearConstraint(A_one, 1, 1),
            LinearConstraint(mem.reshape(1, -1).astype(float), -np.inf, bm),
            LinearConstraint(time.reshape(1, -1), -np.inf, bt)]
    res = milp(risk.reshape(-1), constraints=cons, integrality=np.ones(N * K), bounds=Bounds(0, 1))
    return res


@pytest.mark.parametrize("trial", range(8))
def test_optimum_matches_library_milp_solver(trial):
    N, K = int(RNG.integers(3, 9)), int(RNG.integers(2, 5))
    risk, mem, time, bm, bt = random_instance(N, K)
    rc, x, obj, m, t = oracle.allocate_brute(risk, mem, time, bm, bt)
    res = solve_with_library_milp(risk, mem, time, bm, bt)
    if rc == oracle.ORC_INFEASIBLE:
        assert not res.success
    else:
        assert res.success and obj == pytest.approx(res.fun, abs=1e-7)
        rc2, x2, obj2, *_ = oracle.allocate_dp(risk, mem, time, bm, bt)
        assert rc2 == 0 and obj2 == obj


def test_tiny_config_sized_instance_by_enumeration_and_dp():
    # 8 blocks x 4 configurations = 65,536 assignments, as in the smallest workload
    risk, mem, time, bm, bt = random_instance(8, 4, mem_hi=40)
    a = oracle.allocate_brute(risk, mem, time, bm, bt)
    b = oracle.allocate_dp(risk, mem, time, bm, bt)
    assert a[0] == b[0] == 0 and list(a[1]) == list(b[1])


def test_integer_image():
    risk = np.array([[0.1234567894, 2e7, -3e7, np.inf]])
    mem = np.array([[1, 2, 3, 4]], np.int64); time = np.array([[1.25, 0.0000004, 1.0, 1.0]])
    rc, phi, tau, ok, bt = oracle.integerise(risk, mem, time, 10, 2.5)
    assert rc == 0 and list(phi[0][:3]) == [123456789, 10 ** 15, -10 ** 15] and list(ok[0]) == [1, 1, 1, 0]
    assert list(tau[0][:2]) == [1250000, 0] and bt == 2500000


# ---------------------------------------------------------------- depth-first branch and bound

def _same(a, b):
    assert a[0] == b[0], (a[0], b[0])
    if a[0] == 0:
        assert list(a[1]) == list(b[1]) and a[2:] == b[2:]


@pytest.mark.parametrize("kind", ["real", "int", "flat"])
def test_branch_and_bound_agrees_with_enumeration(kind):
    for trial in range(80):
        N, K = int(RNG.integers(1, 9)), int(RNG.integers(1, 5))
        risk, mem, time, bm, bt = random_instance(N, K, int_risk=(kind == "int"))
        if kind == "flat":
            risk = np.zeros((N, K))
        fb = (RNG.random((N, K)) < 0.15).astype(np.uint8) if trial % 3 == 0 else None
        if trial % 7 == 0:
            risk = risk.copy(); risk[RNG.integers(0, N), RNG.integers(0, K)] = np.nan      # an excluded pair
        _same(oracle.allocate_brute(risk, mem, time, bm, bt, fb), oracle.allocate_bnb(risk, mem, time, bm, bt, fb))


@pytest.mark.parametrize("kind", ["real", "int", "flat"])
def test_branch_and_bound_agrees_with_dynamic_programme(kind):
    for trial in range(15):
        N, K = int(RNG.integers(20, 60)), int(RNG.integers(3, 8))
        risk, mem, time, bm, bt = random_instance(N, K, int_risk=(kind == "int"), mem_hi=12, tau_units=5)
        if kind == "flat":
            risk = np.zeros((N, K))
        _same(oracle.allocate_dp(risk, mem, time, bm, bt), oracle.allocate_bnb(risk, mem, time, bm, bt))


def test_branch_and_bound_special_cases():
    risk = np.array([[0.1, 0.8], [0.3, 0.5]]); mem = np.array([[4, 1], [4, 1]], np.int64); time = np.ones((2, 2))
    rc, x, obj, m, t = oracle.allocate_bnb(risk, mem, time, 5, 10.0)
    assert rc == 0 and list(x) == [0, 1] and obj == pytest.approx(0.6) and m == 5 and t == 2.0
    assert oracle.allocate_bnb(risk, mem, time, 1, 10.0)[0] == oracle.ORC_INFEASIBLE
    assert oracle.allocate_bnb(risk, mem, time, 8, 1.5)[0] == oracle.ORC_INFEASIBLE
    rc, x, *_ = oracle.allocate_bnb(risk, mem, time, 8, 10.0, forbidden=np.array([[1, 0], [0, 0]]))
    assert rc == 0 and list(x) == [1, 0]
    # ties: all assignments with total memory <= 3 cost 0; the smallest vector is (0, 1, 2)
    rc, x, *_ = oracle.allocate_bnb(np.zeros((3, 3)), np.array([[2, 1, 0]] * 3, np.int64), np.ones((3, 3)), 3, 1e6)
    assert rc == 0 and list(x) == [0, 1, 2]
    # slack budgets: per-block arg-min, lowest index on ties
    r = RNG.integers(0, 3, (40, 5)).astype(np.float64)
    rc, x, *_ = oracle.allocate_bnb(r, RNG.integers(0, 9, (40, 5)), np.round(RNG.random((40, 5)) * 4) / 4, 10 ** 9, 1e6)
    assert rc == 0 and list(x) == list(np.argmin(r, axis=1))
    # rows that no assignment meets together although each can be met alone: proved, not guessed
    mem = np.array([[0, 9]] * 6, np.int64); time = np.array([[9.0, 0.0]] * 6)
    assert oracle.allocate_bnb(np.zeros((6, 2)), mem, time, 26, 26.0)[0] == oracle.ORC_INFEASIBLE
    assert oracle.allocate_brute(np.zeros((6, 2)), mem, time, 26, 26.0)[0] == oracle.ORC_INFEASIBLE
    assert oracle.allocate_bnb(np.zeros((6, 2)), mem, time, 27, 27.0)[0] == 0


def test_branch_and_bound_gives_up_rather_than_guess():
    risk, mem, time, _, _ = random_instance(40, 6)
    bm = int(mem.min(1).sum() + 0.5 * (mem.max(1).sum() - mem.min(1).sum()))
    bt = float(time.min(1).sum() + 0.5 * (time.max(1).sum() - time.min(1).sum()))
    rc, *_ = oracle.allocate_bnb(risk, mem, time, bm, bt, node_limit=5)
    assert rc == oracle.ORC_TOO_BIG
    a = oracle.allocate_bnb(risk, mem, time, bm, bt)
    assert a[0] == 0 and oracle.allocate_bnb_nodes() > 5
    _same(oracle.allocate_dp(risk, mem, time, bm, bt), a)
