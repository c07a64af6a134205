"""Pins of the CPU oracle's profiler against what the paper and the mathematics fix:
closed forms, invariants, special cases that reduce to a library routine.
None of these calls the HIP path."""
import math

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(20260504)
BM, BV = float(np.float32(0.9)), float(np.float32(0.999))     # the decay rates are binary32 parameters


def run(gs, **kw):
    b = oracle.Block(gs[0].size, **kw)
    for g in gs:
        b.step(np.asarray(g, np.float32))
    return b


# ---------------------------------------------------------------- Eq. 3 moments

def test_moments_closed_form_weighted_sum():
    T, d = 12, 1000
    gs = [RNG.standard_normal(d).astype(np.float32) for _ in range(T)]
    b = run(gs)
    G = np.stack(gs).astype(np.float64)
    wm = np.array([(1 - BM) * BM ** (T - k) for k in range(1, T + 1)])
    wv = np.array([(1 - BV) * BV ** (T - k) for k in range(1, T + 1)])
    np.testing.assert_allclose(b.m, wm @ G, rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(b.v, wv @ (G * G), rtol=2e-6, atol=1e-10)


@pytest.mark.parametrize("T", [1, 16, 32])
def test_moments_constant_gradient(T):
    g = RNG.standard_normal(513).astype(np.float32)
    b = run([g] * T)
    np.testing.assert_allclose(b.m, (1 - BM ** T) * g.astype(np.float64), rtol=3e-6)
    np.testing.assert_allclose(b.v, (1 - BV ** T) * g.astype(np.float64) ** 2, rtol=3e-6)


def test_snr_constant_gradient_matches_closed_form(golden):
    g = RNG.standard_normal(4096).astype(np.float32)
    for T, val in golden("snr_constant_gradient.txt"):
        st = run([g] * int(T)).finalize()
        assert st.snr == pytest.approx(float(val), rel=5e-5)       # table value: beta_v = 0.999 exactly
        assert st.snr == pytest.approx((1 - BM ** int(T)) ** 2 / (1 - BV ** int(T)), rel=2e-6)


def test_zero_gradient_gives_zero_signals():
    st = run([np.zeros(300, np.float32)] * 3).finalize()
    assert st.snr == 0.0 and st.rho_bar == 0.0 and st.cos_last == 0.0   # NaN cosine -> 0
    assert st.m_sq == 0.0 and st.v_l1 == 0.0
    assert st.A == pytest.approx(0.0, abs=1e-15)                          # log(eps/eps)
    assert st.err_m8 == 0.0 and st.err_v16 == 0.0


def test_bf16_gradient_is_widened_exactly():
    g32 = RNG.standard_normal(700).astype(np.float32)
    bits = (g32.view(np.uint32) >> 16).astype(np.uint16)          # truncation: any bf16 value will do
    wide = (bits.astype(np.uint32) << 16).view(np.float32)
    a, b = oracle.Block(700), oracle.Block(700)
    for _ in range(3):
        a.step(bits); b.step(wide)
    assert np.array_equal(a.m, b.m) and np.array_equal(a.v, b.v) and np.array_equal(a.p, wide)
    assert a.finalize().asdict() == b.finalize().asdict()


# ---------------------------------------------------------------- Eq. 5 direction stability

def test_identical_gradients_rho_is_one():
    g = RNG.standard_normal(2048).astype(np.float32)
    st = run([g] * 5).finalize()
    assert st.rho_bar == pytest.approx(1.0, abs=1e-9) and st.n_cos == 4


def test_alternating_sign_rho_is_minus_one():
    g = RNG.standard_normal(2048).astype(np.float32)
    st = run([g, -g, g, -g]).finalize()
    assert st.rho_bar == pytest.approx(-1.0, abs=1e-9)


def test_disjoint_support_rho_is_zero():
    a = np.zeros(512, np.float32); a[:256] = RNG.standard_normal(256)
    b = np.zeros(512, np.float32); b[256:] = RNG.standard_normal(256)
    assert run([a, b, a, b]).finalize().rho_bar == 0.0


def test_single_step_has_no_cosine():
    st = run([RNG.standard_normal(100).astype(np.float32)]).finalize()
    assert st.rho_bar == 0.0 and st.n_cos == 0 and st.steps == 1


def test_rho_is_ema_of_library_cosines():
    T, d, beta = 9, 3000, 0.9
    base = RNG.standard_normal(d)
    gs = [(base + 0.8 * RNG.standard_normal(d)).astype(np.float32) for _ in range(T)]
    st = run(gs, beta_rho=beta).finalize()
    cs = [float(np.dot(gs[t].astype(np.float64), gs[t - 1].astype(np.float64)) /
                (np.linalg.norm(gs[t].astype(np.float64)) * np.linalg.norm(gs[t - 1].astype(np.float64))))
          for t in range(1, T)]
    rho = cs[0]                       # first cosine initialises the average
    for c in cs[1:]:
        rho = beta * rho + (1 - beta) * c
    assert st.rho_bar == pytest.approx(rho, rel=1e-10)
    assert st.cos_last == pytest.approx(cs[-1], rel=1e-10)
    assert st.g_sq_last == pytest.approx(float(np.dot(gs[-1].astype(np.float64), gs[-1].astype(np.float64))), rel=1e-12)


def test_prescribed_angle():
    e1 = np.zeros(64, np.float32); e1[0] = 1.0
    g2 = np.zeros(64, np.float32); g2[0] = 0.5; g2[1] = math.sqrt(0.75)   # cos = 0.5 (up to fp32 rounding)
    st = run([e1, g2]).finalize()
    assert st.rho_bar == pytest.approx(0.5, abs=1e-7)
    assert st.s_rho == pytest.approx((0.5 - 0.2) / 0.4, abs=1e-6)


# ---------------------------------------------------------------- Eq. 4 anisotropy and the quantile

@pytest.mark.parametrize("d", [1, 2, 3, 10, 11, 257, 5000])
def test_quantile_matches_sort_based_library_quantile(d):
    x = RNG.random(d).astype(np.float32)
    for q in (0.1, 0.9, 0.5):
        assert oracle.quantile(x, q) == pytest.approx(float(np.quantile(x.astype(np.float64), q)), rel=1e-12, abs=1e-300)


def test_equal_magnitudes_have_no_anisotropy():
    g = np.where(RNG.random(1000) < 0.5, -0.37, 0.37).astype(np.float32)
    st = run([g] * 4).finalize()
    assert st.A == pytest.approx(0.0, abs=1e-12) and st.s_A == 0.0


def test_half_scaled_by_ten_saturates_geometry_signal():
    g = np.ones(1000, np.float32); g[::2] = 10.0
    st = run([g] * 3).finalize()
    assert st.A == pytest.approx(math.log(100.0), rel=1e-6) and st.s_A == 1.0


def test_intermediate_geometry_signal():
    g = np.ones(1000, np.float32); g[::2] = 2.0          # v ratio 4 -> A = ln 4
    st = run([g] * 2).finalize()
    assert st.A == pytest.approx(math.log(4.0), rel=1e-6)
    assert st.s_A == pytest.approx((math.log(4.0) - math.log(2.0)) / (math.log(10.0) - math.log(2.0)), rel=1e-6)


def test_constant_sign_scaled_gradient_anisotropy_from_order_statistics():
    kappa = np.exp(0.5 * RNG.standard_normal(20001)).astype(np.float32)
    st = run([kappa] * 6).finalize()
    k2 = kappa.astype(np.float64) ** 2
    want = math.log(np.quantile(k2, 0.9) / np.quantile(k2, 0.1))
    assert st.A == pytest.approx(want, rel=1e-5)
    assert st.q90 / st.q10 == pytest.approx(np.quantile(k2, 0.9) / np.quantile(k2, 0.1), rel=1e-5)


def test_isotropic_noise_anisotropy_is_near_chi_square_baseline(golden):
    d = 200_000
    for T, _lo, _hi, A in golden("chi2_anisotropy.txt"):
        T = int(T)
        if T > 32:
            continue
        gs = [(0.01 * RNG.standard_normal(d)).astype(np.float32) for _ in range(T)]
        assert run(gs).finalize().A == pytest.approx(float(A), abs=0.02)


# ---------------------------------------------------------------- Eq. 8 quantisers

def test_bf16_rounding_matches_library_cast():
    x = np.concatenate([RNG.standard_normal(20000).astype(np.float32) * 10.0 ** RNG.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, np.inf, -np.inf,
                                  1e-40, 2.0 ** -133], np.float32)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.bf16_round(v) for v in x], np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert math.isnan(oracle.bf16_round(float("nan")))


def test_bf16_ties_go_to_even():
    # 1 + 2^-8 lies half way between bf16 neighbours 1 and 1 + 2^-7: even significand wins
    assert oracle.bf16_round(1.0 + 2.0 ** -8) == 1.0
    assert oracle.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6


def test_q8_code_properties():
    assert oracle.q8_code(0.5, 1.0, 127.0) == 64.0          # 63.5 -> even
    assert oracle.q8_code(1.5 / 127.0, 1.0, 127.0) in (1.0, 2.0)
    assert oracle.q8_code(-1.0, 1.0, 127.0) == -127.0
    assert oracle.q8_code(3.0, 3.0, 255.0) == 255.0
    assert oracle.q8_code(1.0, 0.0, 127.0) == 0.0           # empty scale
    assert oracle.q8_code(1e-42, 1e-42, 127.0) == 0.0       # scale overflows -> zero codes
    for k in range(-127, 128):                               # grid points are fixed points
        assert oracle.q8_code(k * 2.0 ** -10, 127 * 2.0 ** -10, 127.0) == float(k)


def test_exactly_representable_states_have_zero_error():
    # beta = 1/2 and power-of-two gradients keep m = (1-2^-t) g, v = (1-2^-t) g^2 within 8 significant bits
    sign = np.where(RNG.random(1024) < 0.5, -1.0, 1.0)
    g = (sign * 2.0 ** RNG.integers(-6, 6, 1024)).astype(np.float32)
    b = run([g] * 6, beta_m=0.5, beta_v=0.5)
    st = b.finalize()
    assert st.err_m16 == 0.0 and st.err_v16 == 0.0
    assert st.Q16 == pytest.approx(1.0, abs=1e-11) and st.lQ16 == pytest.approx(0.0, abs=1e-11)
    # 8 bit: all magnitudes in a group equal -> every code is +-127 / 255 -> exact
    g = (sign * 0.3).astype(np.float32)
    st = run([g] * 3).finalize()
    assert st.err_m8 == pytest.approx(0.0, abs=1e-15) and st.err_v8 == pytest.approx(0.0, abs=1e-15)
    assert st.Q8 == pytest.approx(1.0, abs=1e-11)


def test_first_moment_on_the_8bit_grid_is_exact():
    # T = 1, beta_m = 1/2: m = g/2. Put m on the grid k a/127 with a = 127 2^-10.
    k = RNG.integers(-127, 128, 512); k[0] = 127; k[256] = -127      # both groups share a = 127 2^-10
    g = (2.0 * k * 2.0 ** -10).astype(np.float32)
    st = run([g], beta_m=0.5).finalize()
    assert st.err_m8 == 0.0 and st.err_v8 > 0.0


def test_quantiser_error_bounds_and_uniform_noise_level():
    d, qb = 256 * 64, 256
    m_target = RNG.uniform(-1.0, 1.0, d)
    g = (2.0 * m_target).astype(np.float32)                  # T = 1, beta_m = beta_v = 1/2
    b = run([g], beta_m=0.5, beta_v=0.5)
    st = b.finalize()
    m, v = b.m.astype(np.float64), b.v.astype(np.float64)
    am = np.abs(m).reshape(-1, qb).max(1); av = v.reshape(-1, qb).max(1)
    step_m, step_v = am / 127.0, av / 255.0
    Em = (st.err_m8 * math.sqrt(st.m_sq)) ** 2
    Ev = (st.err_v8 * np.linalg.norm(v)) ** 2
    assert Em <= qb * np.sum((step_m / 2) ** 2) * (1 + 1e-9)
    assert Ev <= qb * np.sum((step_v / 2) ** 2) * (1 + 1e-9)
    assert Em == pytest.approx(qb * np.sum(step_m ** 2) / 12.0, rel=0.05)    # uniform rounding noise
    # bf16 keeps 8 significant bits: spacing 2^(e-7) in the binade of 2^e, so each element is off by
    # at most 2^(e-8) (relative error <= 2^-8) and by 2^(e-8)/sqrt(3) in the root mean square
    assert st.err_m16 <= 2.0 ** -8 and st.err_v16 <= 2.0 ** -8
    binade = 2.0 ** np.floor(np.log2(np.abs(m)))
    assert st.err_m16 == pytest.approx(2.0 ** -8 / math.sqrt(3.0) * math.sqrt(np.mean(binade ** 2) / np.mean(m * m)), rel=0.05)


def test_Q16_matches_library_cast_and_library_cosine():
    T, d = 7, 4096
    gs = [RNG.standard_normal(d).astype(np.float32) * 0.01 for _ in range(T)]
    b = run(gs)
    st = b.finalize()
    m, v = torch.from_numpy(b.m), torch.from_numpy(b.v)
    m16 = m.to(torch.bfloat16).to(torch.float64).numpy(); v16 = v.to(torch.bfloat16).to(torch.float64).numpy()
    u32 = b.m.astype(np.float64) / (np.sqrt(b.v.astype(np.float64)) + 1e-8)
    u16 = m16 / (np.sqrt(v16) + 1e-8)
    cos = float(u32 @ u16 / (np.linalg.norm(u32) * np.linalg.norm(u16)))
    assert 1.0 - st.Q16 == pytest.approx(1.0 - cos, rel=1e-6)
    assert st.lQ16 == pytest.approx(-math.log(cos), rel=1e-5)
    assert st.lQ32 == pytest.approx(0.0, abs=3e-12)
    assert st.err_m16 == pytest.approx(np.linalg.norm(m16 - b.m) / (np.linalg.norm(b.m.astype(np.float64)) + 1e-12), rel=1e-9)
    assert st.err_v16 == pytest.approx(np.linalg.norm(v16 - b.v) / (np.linalg.norm(b.v.astype(np.float64)) + 1e-12), rel=1e-9)


def test_Q8_two_level_closed_form():
    # v constant (|g| constant) -> v8 = v; m takes the group maximum a on half the coordinates and
    # 0.4 a/127 (code 0) on the rest -> Q8 = 1 / sqrt(1 + (0.4/127)^2), whatever the scale.
    # T = 1 cannot separate m from v, so use two steps: g1 = c, g2 = +-c keeps v = const * c^2.
    d = 512
    c = 0.25
    g1 = np.full(d, c, np.float32)
    # after two steps with beta_m = 1/2: m = g1/4 + g2/2.  g2 = c -> m = 0.75 c ; g2 = -c -> m = -0.25 c
    g2 = np.full(d, c, np.float32); g2[1::2] = -c
    st = run([g1, g2], beta_m=0.5).finalize()
    # codes: 127 for 0.75c; rint(-127/3) = -42 for -0.25c -> m8 = -42/127 * 0.75 c
    q_small = -42.0 / 127.0 * 0.75
    num = 0.75 * 0.75 + (-0.25) * q_small
    den = math.sqrt(0.75 ** 2 + 0.25 ** 2) * math.sqrt(0.75 ** 2 + q_small ** 2)
    assert st.Q8 == pytest.approx(num / den, rel=1e-9)
    assert st.err_v8 == pytest.approx(0.0, abs=1e-15)
    assert st.err_m8 == pytest.approx(abs(-0.25 - q_small) / math.sqrt(0.75 ** 2 + 0.25 ** 2), rel=1e-9)


def test_zero_second_moment_code_blows_up_the_8bit_direction():
    # one large coordinate per group pushes every other v below half a code: v8 = 0 there and
    # u8 = m8 / eps_u, so the 8-bit direction is dominated by those coordinates
    g = np.full(256, 1e-3, np.float32); g[0] = 1.0
    st = run([g] * 2).finalize()
    assert st.Q8 < 0.2 and st.lQ8 > 1.0 and st.Q16 > 0.99999


def test_power_of_two_rescaling_is_invariant():
    T, d = 5, 2048
    gs = [RNG.standard_normal(d).astype(np.float32) for _ in range(T)]
    a = run(gs).finalize()
    b = run([g * np.float32(2.0 ** 7) for g in gs]).finalize()
    for f in ("rho_bar", "A", "snr", "Q16", "Q8", "err_m16", "err_v16", "err_m8", "err_v8"):
        assert getattr(a, f) == pytest.approx(getattr(b, f), rel=1e-6), f
    assert b.m_sq == pytest.approx(a.m_sq * 2.0 ** 14, rel=1e-12)


# ---------------------------------------------------------------- quantisation groups / segments

def test_splitting_at_a_group_boundary_adds_raw_sums():
    T, d, cut = 4, 256 * 5 + 77, 256 * 2
    gs = [RNG.standard_normal(d).astype(np.float32) for _ in range(T)]
    whole = run(gs); left = run([g[:cut] for g in gs]); right = run([g[cut:] for g in gs])
    sw, sl, sr = whole.finalize(), left.finalize(), right.finalize()
    assert sw.m_sq == pytest.approx(sl.m_sq + sr.m_sq, rel=1e-12)
    assert sw.v_l1 == pytest.approx(sl.v_l1 + sr.v_l1, rel=1e-12)
    Em = lambda s: (s.err_m8 * math.sqrt(s.m_sq)) ** 2
    assert Em(sw) == pytest.approx(Em(sl) + Em(sr), rel=1e-9)
    # an off-boundary cut regroups the coordinates and changes the 8-bit error
    l2 = run([g[:cut + 3] for g in gs]).finalize(); r2 = run([g[cut + 3:] for g in gs]).finalize()
    assert abs(Em(sw) - Em(l2) - Em(r2)) > 1e-6 * Em(sw)


def test_permuting_whole_groups_changes_nothing_but_free_permutation_changes_8bit_terms():
    T, d = 3, 256 * 6
    gs = [(RNG.standard_normal(d) * np.exp(RNG.standard_normal(d))).astype(np.float32) for _ in range(T)]
    perm_g = np.concatenate([np.arange(256) + 256 * k for k in RNG.permutation(6)])
    perm_f = RNG.permutation(d)
    a = run(gs).finalize(); b = run([g[perm_g] for g in gs]).finalize(); c = run([g[perm_f] for g in gs]).finalize()
    for f in oracle.STAT_FIELDS:
        assert getattr(a, f) == pytest.approx(getattr(b, f), rel=1e-11, abs=1e-14), f
    for f in ("rho_bar", "snr", "A", "Q16", "err_m16", "err_v16"):
        assert getattr(a, f) == pytest.approx(getattr(c, f), rel=1e-11), f
    assert abs(a.err_m8 - c.err_m8) > 1e-6 * a.err_m8


def test_blocks_are_independent():
    blocks = [(0, 300), (320, 1000), (1400, 64)]
    flat = [RNG.standard_normal(1500).astype(np.float32) for _ in range(3)]
    p = oracle.Profiler(blocks)
    for f in flat:
        p.step(f)
    other = [f.copy() for f in flat]
    for f in other:
        f[:320] = 7.0; f[1320:] = -3.0
    q = oracle.Profiler(blocks)
    for f in other:
        q.step(f)
    assert p.state[1].finalize().asdict() == q.state[1].finalize().asdict()


# ---------------------------------------------------------------- non-finite second moments in the quantile (Eq. 4)

def test_quantile_ranks_nan_above_infinity_like_a_library_sort():
    """numpy.sort places NaN after +inf; the order statistics the oracle interpolates between must be the
    same ones, whatever mixture of finite values, +inf and NaN the block holds."""
    def library(x, q):
        s = np.sort(x.astype(np.float64))
        pos = q * (s.size - 1); lo = int(math.floor(pos)); hi = min(lo + 1, s.size - 1)
        with np.errstate(invalid="ignore"):
            return s[lo] + (pos - lo) * (s[hi] - s[lo])
    for trial in range(40):
        d = int(RNG.integers(5, 400))
        x = (RNG.standard_normal(d) ** 2).astype(np.float32)
        n_inf, n_nan = int(RNG.integers(0, max(1, d // 4))), int(RNG.integers(0, max(1, d // 4)))
        where = RNG.permutation(d)
        x[where[:n_inf]] = np.inf
        x[where[n_inf:n_inf + n_nan]] = np.nan
        for q in (0.0, 0.1, 0.5, 0.9, 1.0, float(RNG.random())):
            got, want = oracle.quantile(x, q), library(x, q)
            assert (np.isnan(got) and np.isnan(want)) or got == want, (trial, d, n_inf, n_nan, q, got, want)
    # the cases spelled out: NaN is the largest, +inf the next (an infinite or NaN neighbour turns the
    # interpolated value into NaN even at weight 0, as IEEE arithmetic has it: 0 * inf)
    x = np.array([3.0, np.nan, 1.0, np.inf, 2.0], np.float32)          # ascending: 1 2 3 inf nan
    assert oracle.quantile(x, 0.0) == 1.0 and oracle.quantile(x, 0.25) == 2.0 and oracle.quantile(x, 0.375) == 2.5
    assert np.isnan(oracle.quantile(x, 0.5)) and np.isnan(oracle.quantile(x, 1.0))
    assert oracle.quantile(np.array([np.nan, 5.0, 7.0], np.float32), 0.0) == 5.0
    assert oracle.quantile(np.array([np.inf, np.nan, 5.0, 7.0, 6.0], np.float32), 0.25) == 6.0


# ---------------------------------------------------------------- the fixed fp32 state sequence against the plain fp64 definitions

def _round_to_significand(x, bits):
    m, e = np.frexp(x)
    return np.ldexp(np.rint(m * 2.0 ** bits) / 2.0 ** bits, e)         # nearest, ties to even, no exponent limits


def _definitions_in_fp64(gs, qb=256, eps=1e-12):
    """Eq. 3, Eq. 4, Eq. 5 (right) and Eq. 8 evaluated in fp64 throughout: states advanced as
    beta x + (1 - beta) y, 8-bit codes decided as rint(L x / a) in fp64, bf16 as the nearest 8-bit significand."""
    eu = float(np.float32(1e-8))
    d = gs[0].size
    m, v = np.zeros(d), np.zeros(d)
    for g in gs:
        g = g.astype(np.float64)
        m = BM * m + (1 - BM) * g
        v = BV * v + (1 - BV) * g * g
    out = {}
    S_mm, S_v1, S_vv = float((m * m).sum()), float(v.sum()), float((v * v).sum())
    out["m_sq"], out["v_l1"], out["snr"] = S_mm, S_v1, S_mm / (S_v1 + eps)
    out["q10"], out["q90"] = (float(np.quantile(v, q)) for q in (0.1, 0.9))
    out["A"] = math.log((out["q90"] + eps) / (out["q10"] + eps))
    code_m, code_v = np.zeros(d), np.zeros(d)
    m8, v8 = np.zeros(d), np.zeros(d)
    for s in range(0, d, qb):
        sl = slice(s, min(d, s + qb))
        am, av = np.abs(m[sl]).max(), v[sl].max()
        if am > 0:
            code_m[sl] = np.rint(127 * m[sl] / am); m8[sl] = am * code_m[sl] / 127
        if av > 0:
            code_v[sl] = np.rint(255 * v[sl] / av); v8[sl] = av * code_v[sl] / 255
    m16, v16 = _round_to_significand(m, 8), _round_to_significand(v, 8)
    u32 = m / (np.sqrt(v) + eu)
    for tag, mq, vq in (("16", m16, v16), ("8", m8, v8)):
        ub = mq / (np.sqrt(vq) + eu)
        q = float((u32 * ub).sum() / (math.sqrt((u32 * u32).sum()) * math.sqrt((ub * ub).sum()) + eps))
        out["Q" + tag] = min(max(q, eps), 1.0)
        out["lQ" + tag] = -math.log(out["Q" + tag] + eps)
        out["err_m" + tag] = math.sqrt(((mq - m) ** 2).sum()) / (math.sqrt(S_mm) + eps)
        out["err_v" + tag] = math.sqrt(((vq - v) ** 2).sum()) / (math.sqrt(S_vv) + eps)
    return out, code_m, code_v, m16, v16


def test_fp32_state_sequence_stays_close_to_the_fp64_definitions():
    """The oracle advances m, v in one fixed fp32 sequence and decides the 8-bit codes in fp32 (so that the
    kernels can be compared bit for bit).  Measured against the same definitions in fp64 throughout, on the
    ragged layout's stream: every reported statistic moves by less than a fifth of the parity tolerance
    (largest seen: 9e-6 relative, the bf16 error of v on a 4,099-coordinate block), including the blocks
    where a quantiser decision flips between the two evaluations."""
    from synth import gradgen, workloads as W
    w = W.ragged("f32", 1)
    flipped, worst = [], 0.0
    for i, b in enumerate(w.blocks):
        gs = [gradgen.block_gradient(5, i, b, t) for t in range(1, w.T + 1)]
        ob = run(gs)
        st = ob.finalize()
        ref, code_m, code_v, m16, v16 = _definitions_in_fp64(gs)
        om, ov = ob.m, ob.v
        flips = 0
        for s in range(0, b.numel, 256):
            sl = slice(s, min(b.numel, s + 256))
            am, av = float(np.abs(om[sl]).max()), float(ov[sl].max())
            flips += sum(oracle.q8_code(x, am, 127.0) != k for x, k in zip(om[sl], code_m[sl]))
            flips += sum(oracle.q8_code(x, av, 255.0) != k for x, k in zip(ov[sl], code_v[sl]))
        flips += int((m16 != np.array([oracle.bf16_round(x) for x in om])).sum())
        flips += int((v16 != np.array([oracle.bf16_round(x) for x in ov])).sum())
        if flips:
            flipped.append((b.name, b.numel, flips))
        for k, r in ref.items():
            shift = abs(getattr(st, k) - r) / (1e-6 + 1e-4 * abs(r))      # 1.0 = the parity tolerance
            worst = max(worst, shift)
            assert shift < 0.2, (b.name, b.numel, k, getattr(st, k), r)
    # decisions do flip now and then (a value within an fp32 rounding of a code boundary); they are rare and,
    # by the assertion above, invisible in the statistics even on the 1-, 3- and 5-coordinate blocks
    assert len(flipped) <= 4 and all(n >= 1000 and f <= max(3, n // 5000) for _, n, f in flipped), flipped
    assert 0.0 < worst < 0.2
