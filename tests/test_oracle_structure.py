"""Pins of the oracle's structure residual (Eq. 7) and distortion (Eq. 6)."""
import math

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(77)
BV = float(np.float32(0.999))


def block_with_v_from(g, T=1, **kw):
    b = oracle.Block(g.size, **kw)
    for _ in range(T):
        b.step(np.ascontiguousarray(g, np.float32).ravel())
    return b


def test_rank_one_second_moment_has_no_residual():
    a, c = np.exp(RNG.standard_normal(37)), np.exp(RNG.standard_normal(53))
    b = block_with_v_from(np.outer(a, c), T=3)
    assert b.structure_residual(37, 53) == pytest.approx(0.0, abs=3e-7)       # fp32 rounding of v only
    assert block_with_v_from(np.full((8, 9), 0.3)).structure_residual(8, 9) == pytest.approx(0.0, abs=1e-7)


def test_identity_pattern_worked_by_hand():
    # S proportional to I_2: r = c = (1/2, 1/2) S11, mu = S11/2, S~ = S11/2 everywhere
    # |S - S~|^2 = 4 (S11/2)^2, |S|^2 = 2 S11^2  ->  F = 1/sqrt(2)
    b = block_with_v_from(np.eye(2))
    assert b.structure_residual(2, 2) == pytest.approx(1.0 / math.sqrt(2.0), rel=1e-8)
    # n x n identity: S~ = S11/n everywhere: F^2 = (n (1-1/n)^2 + (n^2-n)/n^2) / n = (n-1)/n
    b = block_with_v_from(np.eye(5))
    assert b.structure_residual(5, 5) == pytest.approx(math.sqrt(4.0 / 5.0), rel=1e-8)


def test_matches_library_outer_product_and_frobenius_norm():
    R, C_ = 41, 67
    g = RNG.standard_normal((R, C_)) * np.exp(RNG.standard_normal((R, 1))) * np.exp(0.5 * RNG.standard_normal((1, C_)))
    b = block_with_v_from(g, T=2)
    S = b.v.astype(np.float64).reshape(R, C_)
    St = np.outer(S.mean(1), S.mean(0)) / S.mean()
    want = np.linalg.norm(S - St, "fro") / (np.linalg.norm(S, "fro") + 1e-12)
    assert b.structure_residual(R, C_) == pytest.approx(want, rel=1e-12)
    # transposition and scale leave F unchanged
    bt = block_with_v_from(g.T.copy(), T=2)
    assert bt.structure_residual(C_, R) == pytest.approx(want, rel=1e-6)
    bs = block_with_v_from(g * 2.0 ** 5, T=2)
    assert bs.structure_residual(R, C_) == pytest.approx(want, rel=1e-6)


def test_isotropic_noise_residual_is_near_chi_square_level():
    # T = 1: S = (1-beta_v) g^2, g ~ N(0,1): E S = 1, Var S = 2 (in units of (1-beta_v)), no structure:
    # F -> sqrt(Var / E S^2) = sqrt(2/3)
    b = block_with_v_from(RNG.standard_normal((300, 400)))
    assert b.structure_residual(300, 400) == pytest.approx(math.sqrt(2.0 / 3.0), abs=0.01)
    # equal-weight window of T steps: S ~ chi2_T / T: F -> sqrt(2 / (T + 2))
    bb = oracle.Block(300 * 400)
    for _ in range(8):
        bb.step(RNG.standard_normal(300 * 400).astype(np.float32))
    assert bb.structure_residual(300, 400) == pytest.approx(math.sqrt(2.0 / 10.0), abs=0.01)


def test_non_matrix_blocks_and_zero_state():
    b = block_with_v_from(RNG.standard_normal(100))
    assert b.structure_residual(0, 0) == 0.0 and b.structure_residual(7, 9) == 0.0
    z = block_with_v_from(np.zeros((4, 5)))
    assert z.structure_residual(4, 5) == 0.0


def test_structure_signal_enters_the_risk_of_factored_configurations():
    b = block_with_v_from(RNG.standard_normal((30, 40)))
    F = b.structure_residual(30, 40)
    st = b.finalize(F_raw=F)
    assert st.F == F and st.s_F == pytest.approx(min(F, 1.0))
    assert oracle.phi(st, (1, 0, 0, 1, 32)) - oracle.phi(st, (1, 0, 0, 0, 32)) == pytest.approx(st.s_F + 0.1, rel=1e-12)


# ---------------------------------------------------------------- Eq. 6 distortion

def test_uniform_preconditioner_has_no_distortion():
    g = np.where(RNG.random(500) < 0.5, -0.2, 0.2)           # |g| constant -> v constant -> p = p-bar
    b = block_with_v_from(g, T=4)
    assert b.distortion(RNG.standard_normal(500).astype(np.float32)) == pytest.approx(0.0, abs=1e-12)


def test_two_level_preconditioner_closed_form():
    # half the coordinates have sqrt(v) = s, the other half 3 s: p = 1/s, 1/(3s); p-bar = 2/(3s);
    # p/p-bar - 1 = +1/2, -1/2  ->  C = 1/2 for any theta
    g = np.ones(400); g[200:] = 3.0
    b = block_with_v_from(g)
    theta = RNG.standard_normal(400).astype(np.float32)
    assert b.distortion(theta) == pytest.approx(0.5, rel=1e-6)
    # weighting by theta: theta supported on the first half only sees +1/2
    theta[200:] = 0
    assert b.distortion(theta) == pytest.approx(0.5, rel=1e-6)


def test_distortion_matches_library_norms_and_is_scale_free_in_theta():
    g = RNG.standard_normal(3000) * np.exp(RNG.standard_normal(3000))
    b = block_with_v_from(g, T=3)
    theta = RNG.standard_normal(3000).astype(np.float32)
    p = 1.0 / (np.sqrt(b.v.astype(np.float64)) + 1e-12)
    want = np.linalg.norm((p / p.mean() - 1.0) * theta) / (np.linalg.norm(theta.astype(np.float64)) + 1e-12)
    assert b.distortion(theta) == pytest.approx(want, rel=1e-12)
    assert b.distortion(theta * 8) == pytest.approx(want, rel=1e-9)
    st = b.finalize(C_raw=want)
    assert st.C == want and st.C_tilde == pytest.approx(math.log1p(want), rel=1e-15)
    bits = (theta.view(np.uint32) >> 16).astype(np.uint16)                  # bf16 parameters are widened exactly
    wide = (bits.astype(np.uint32) << 16).view(np.float32)
    assert b.distortion(bits) == b.distortion(wide)
