"""HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

import oracle
from oracle.runner import (OracleRunner, assert_risk_close, assert_stats_close, oracle_params, to_host_bits)
from synth import workloads as W

pytestmark = pytest.mark.gpu
SEED = 1


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2605_04711_amd as B
    from paper_2605_04711_amd import binding
    from synth import device
    B.load_library(); device.lib()
    return dict(torch=torch, B=B, binding=binding, device=device)


def run_both(env, w, T, only=None, chunk_groups=0, check_state=True, seed=SEED, theta_dtype=None, **shape):
    torch, binding, device = env["torch"], env["binding"], env["device"]
    params = binding.default_profile_params(grad_dtype=1 if w.grad_dtype == "bf16" else 0, chunk_groups=chunk_groups, **shape)
    prof = binding.Profiler(w.blocks, params)
    orc = OracleRunner(w.blocks, only, **oracle_params(params))
    buf = device.new_buffer(w)
    for t in range(1, T + 1):
        device.fill(w, buf, seed, t)
        prof.step(buf)
        orc.step_from_device(buf)
    theta = None
    if theta_dtype is not None:                              # parameters for Eq. 6, same layout as the gradients
        gen = torch.Generator(device="cuda:0"); gen.manual_seed(1234 + seed)
        theta = (0.02 * torch.randn(w.buffer_numel, device="cuda:0", generator=gen)).to(theta_dtype)
    stats, risk = prof.finalize(w.configs, theta=theta)
    ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in w.blocks], theta=theta)
    for row, i in enumerate(orc.only):
        assert_stats_close(stats[i], ostats[i], f"{w.name} block {i} ({w.blocks[i].name}, d={w.blocks[i].numel})")
        assert_risk_close(risk[i], orisk[row], f"{w.name} block {i}")
        if check_state:
            m, v, p = prof.state(i)
            ob = orc.state[i]
            assert np.array_equal(to_host_bits(m).view(np.uint32), ob.m.view(np.uint32)), f"m bits, block {i}"
            assert np.array_equal(to_host_bits(v).view(np.uint32), ob.v.view(np.uint32)), f"v bits, block {i}"
            gp = to_host_bits(p)
            want = ob.p if gp.dtype == np.float32 else (ob.p.view(np.uint32) >> 16).astype(np.uint16)
            assert np.array_equal(gp.view(want.dtype), want), f"g_prev bits, block {i}"
    torch.cuda.synchronize()
    return prof, stats, risk, ostats, orisk


def test_tiny_all_blocks_all_steps_and_allocation(env):
    B = env["B"]
    w = W.make("tiny")
    prof, stats, risk, ostats, orisk = run_both(env, w, w.T)
    mem, tc, bm, cap = W.allocation_inputs(w)
    cap = 1e9 if not np.isfinite(cap) else cap
    x, obj, m, t = B.allocate(risk, mem, tc, bm, cap)
    rc, ox, oobj, om, ot = oracle.allocate_brute(risk, mem, tc, bm, cap)          # same risk table: bit exact
    assert rc == 0 and list(x) == list(ox) and obj == oobj and m == om and t == ot
    rc, ox2, *_ = oracle.allocate_brute(orisk, mem, tc, bm, cap)
    assert rc == 0 and m <= bm


def test_tiny_bf16_gradients(env):
    w = W.make("tiny"); w.grad_dtype = "bf16"
    run_both(env, w, 6, theta_dtype=env["torch"].bfloat16)


ragged_workload = W.ragged


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pad,chunk_groups,reverse", [(1, 2, False), (64, 0, True), (3, 1, False)])
def test_ragged_blocks_unaligned_offsets_gaps_and_order(env, dtype, pad, chunk_groups, reverse):
    torch = env["torch"]
    run_both(env, ragged_workload(dtype, pad, reverse), 5, chunk_groups=chunk_groups,
             theta_dtype=torch.float32 if dtype == "f32" else torch.bfloat16)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    dict(groups_per_wave=1, waves_per_workgroup=4, resident_workgroups=8),
    dict(groups_per_wave=2, waves_per_workgroup=4, resident_workgroups=3),
    dict(groups_per_wave=2, waves_per_workgroup=4, chunk_groups=3, resident_workgroups=5),
    dict(groups_per_wave=1, waves_per_workgroup=4, chunk_groups=9),                      # several rounds per slice
    dict(groups_per_wave=2, waves_per_workgroup=4, chunk_groups=20, chunk_slices=1),     # 8 + 8 + 4 groups
    dict(groups_per_wave=2, waves_per_workgroup=4, chunk_groups=1, resident_workgroups=4),
    dict(groups_per_wave=2, waves_per_workgroup=1, chunk_groups=4, resident_workgroups=10),
    dict(groups_per_wave=1, waves_per_workgroup=1, chunk_groups=7, chunk_slices=3, resident_workgroups=32),   # slices of 3, 3, 1
    dict(groups_per_wave=2, waves_per_workgroup=2, chunk_groups=16, chunk_slices=16),    # slices shorter than a round
    dict(groups_per_wave=1, waves_per_workgroup=2, chunk_groups=5, chunk_slices=64, resident_workgroups=16),
])
def test_launch_shapes_leave_the_results_alone(env, dtype, shape):
    """Chunks of one slice and of several, slices of one round, of several and of a partial one, one or two groups
    per wavefront, 1, 2 or 4 wavefronts per workgroup, limited and unlimited residency: the same statistics and
    bit-identical states."""
    run_both(env, ragged_workload(dtype, 1), 4, theta_dtype=env["torch"].float32, **shape)


def check_allocation(env, w, risk):
    """The GPU-produced risk table through both solvers of Eq. 2: same answer, bit for bit."""
    B = env["B"]
    mem, tc, bm, cap = W.allocation_inputs(w)
    cap = 1.3 * len(w.blocks) if not np.isfinite(cap) else cap
    x, obj, m, t = B.allocate(risk, mem, tc, bm, cap)
    rc, ox, oobj, om, ot = oracle.allocate_bnb(risk, mem, tc, bm, cap)
    assert rc == 0 and list(x) == list(ox) and (obj, m, t) == (oobj, om, ot), w.name
    assert m <= bm and t <= cap + 1e-9


def test_resnet50_all_blocks_all_steps(env):
    w = W.make("resnet50")
    prof, stats, risk, ostats, orisk = run_both(env, w, w.T, theta_dtype=env["torch"].float32)
    check_allocation(env, w, risk)


def test_gpt2_small_all_steps(env):
    w = W.make("gpt2_small")
    only = [i for i, b in enumerate(w.blocks) if b.numel < 3_000_000]          # everything but the two embeddings
    run_both(env, w, w.T, only=only, check_state=False)


def test_gpt2_small_embeddings_heavy_tailed(env):
    w = W.make("gpt2_small")
    run_both(env, w, 4, only=[0, 1])


def test_full_candidate_space_with_soft_preference(env):
    """21 candidates (Sec. 4.1) and the soft preference of Sec. 3.2 in the risk table."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = W.make("tiny")
    k21 = W.k21()
    pref = [1 if n.startswith("adamw") else 0 for n in k21["config_names"]]
    prof = binding.Profiler(w.blocks)
    orc = OracleRunner(w.blocks, **oracle_params(prof.params))
    buf = device.new_buffer(w)
    for t in range(1, 6):
        device.fill(w, buf, 2, t); prof.step(buf); orc.step_from_device(buf)
    rp = binding.default_risk_params(lambda_pref=0.3, gamma=0.2)
    stats, risk = prof.finalize(k21["configs"], risk_params=rp, pref_mask=pref)
    orp = oracle.default_risk_params(lambda_pref=0.3, gamma=0.2)
    ostats, orisk = orc.finalize(k21["configs"], rp=orp, pref_mask=pref, shapes=[(b.rows, b.cols) for b in w.blocks])
    assert risk.shape == (8, 21)
    assert_risk_close(risk, orisk, "k21")


@pytest.mark.parametrize("kw", [dict(A_low=0.8 * np.log(2.0), A_high=1.2 * np.log(10.0)), dict(A_low=1.2 * np.log(2.0), A_high=0.8 * np.log(10.0)),
                                dict(rho_low=0.0, rho_high=1.0, eta_low=-1.0, eta_high=4.0), dict(use_snr_gate=0, gamma=0.0), dict(gamma=1.0)])
def test_risk_parameters_away_from_the_defaults(env, kw):
    """Anchors of App. A moved (the +-20 % of the paper's anchor study among them), SNR gate off, other gamma."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload("f32", 64)
    prof = binding.Profiler(w.blocks)
    orc = OracleRunner(w.blocks, **oracle_params(prof.params))
    buf = device.new_buffer(w)
    for t in range(1, 5):
        device.fill(w, buf, 8, t); prof.step(buf); orc.step_from_device(buf)
    theta = torch.randn(w.buffer_numel, device="cuda:0")
    stats, risk = prof.finalize(w.configs, risk_params=binding.default_risk_params(**kw), theta=theta)
    ostats, orisk = orc.finalize(w.configs, rp=oracle.default_risk_params(**kw), shapes=[(b.rows, b.cols) for b in w.blocks], theta=theta)
    for i in range(len(w.blocks)):
        assert_stats_close(stats[i], ostats[i], f"block {i}")
    assert_risk_close(risk, orisk, str(kw))


def test_steps_and_finalize_on_a_side_stream(env):
    """Generation, step and finalize are ordered by one non-default stream alone (default priority)."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload("bf16", 64)
    params = binding.default_profile_params(grad_dtype=1)
    side = torch.cuda.Stream()
    bufs = [device.new_buffer(w) for _ in range(4)]
    torch.cuda.synchronize()
    prof = binding.Profiler(w.blocks, params)
    with torch.cuda.stream(side):
        for t, buf in enumerate(bufs, start=1):
            device.fill(w, buf, 31, t)                   # launched on the current (side) stream
            prof.step(buf, stream=side)
        stats, risk = prof.finalize(w.configs, stream=side)
    side.synchronize()
    orc = OracleRunner(w.blocks, None, **oracle_params(params))
    for buf in bufs:
        orc.step_from_device(buf)
    ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in w.blocks])
    for i in range(len(w.blocks)):
        assert_stats_close(stats[i], ostats[i], f"side stream block {i}")
    assert_risk_close(risk, orisk, "side stream")


@pytest.mark.parametrize("dtype,shape", [("f32", dict()), ("bf16", dict()), ("bf16", dict(chunk_groups=3, groups_per_wave=2)),
                                         ("f32", dict(chunk_groups=20, groups_per_wave=1))])
def test_nothing_is_written_outside_the_workspace(env, dtype, shape):
    """Guard bands of 1 MiB before and after the workspace (and after the gradient and parameter buffers) keep
    their pattern through begin, steps and finalize with F and C."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload(dtype, 3)
    params = binding.default_profile_params(grad_dtype=1 if dtype == "bf16" else 0, **shape)
    nbytes = binding.workspace_bytes(w.blocks, params)
    band = 1 << 20
    arena = torch.full((band + nbytes + band,), 0xA5, dtype=torch.uint8, device="cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gbuf = torch.full((w.buffer_numel + band,), 1.0, dtype=tdt, device="cuda:0")
    theta = torch.full((w.buffer_numel + band,), 0.5, dtype=tdt, device="cuda:0")
    prof = binding.Profiler(w.blocks, params, workspace=arena[band:band + nbytes])
    for t in range(1, 4):
        device.fill(w, gbuf[:w.buffer_numel], 13, t)
        prof.step(gbuf[:w.buffer_numel])
    prof.finalize(w.configs, theta=theta[:w.buffer_numel])
    torch.cuda.synchronize()
    assert bool((arena[:band] == 0xA5).all()) and bool((arena[band + nbytes:] == 0xA5).all())
    assert bool((gbuf[w.buffer_numel:] == 1.0).all()) and bool((theta[w.buffer_numel:] == 0.5).all())
    prof.close()


def test_dirty_workspace_and_windows_back_to_back(env):
    """begin must not depend on what the workspace held: it is filled with 0xFF bytes (NaN patterns) first,
    then reused for a second window after end; finalize in the middle of a window leaves the window intact."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload("bf16", 3)
    params = binding.default_profile_params(grad_dtype=1)
    ws = torch.full((binding.workspace_bytes(w.blocks, params) + 4096,), 0xFF, dtype=torch.uint8, device="cuda:0")
    shapes = [(b.rows, b.cols) for b in w.blocks]
    buf = device.new_buffer(w)
    for window, (seed, T) in enumerate([(11, 5), (12, 3)]):
        prof = binding.Profiler(w.blocks, params, workspace=ws)
        orc = OracleRunner(w.blocks, None, **oracle_params(params))
        for t in range(1, T + 1):
            device.fill(w, buf, seed, t)
            prof.step(buf)
            orc.step_from_device(buf)
            if t == 2:                                       # a look at the statistics in mid-window
                stats, _ = prof.finalize()
                ostats, _ = orc.finalize(w.configs, shapes=shapes)
                for i in range(len(w.blocks)):
                    assert_stats_close(stats[i], ostats[i], f"window {window} mid block {i}")
        stats, risk = prof.finalize(w.configs)
        ostats, orisk = orc.finalize(w.configs, shapes=shapes)
        for i in range(len(w.blocks)):
            assert_stats_close(stats[i], ostats[i], f"window {window} block {i}")
            assert_risk_close(risk[i], orisk[i], f"window {window} block {i}")
            m, v, _ = prof.state(i)
            assert np.array_equal(to_host_bits(m).view(np.uint32), orc.state[i].m.view(np.uint32))
            assert np.array_equal(to_host_bits(v).view(np.uint32), orc.state[i].v.view(np.uint32))
        prof.close()


def test_two_runs_give_identical_bits(env):
    w = ragged_workload("f32", 1)
    a = run_both(env, w, 4, chunk_groups=2)[1]
    b = run_both(env, w, 4, chunk_groups=2)[1]
    assert bytes(a) == bytes(b)


def test_constant_gradient_direction_is_one_and_snr_closed_form(env):
    torch, binding = env["torch"], env["binding"]
    n = 100_003
    g = torch.randn(n, device="cuda:0")
    prof = binding.Profiler([(0, n)])
    for _ in range(16):
        prof.step(g)
    st = prof.finalize()[0][0]
    bm, bv = float(np.float32(0.9)), float(np.float32(0.999))
    assert st.rho_bar == pytest.approx(1.0, abs=1e-9)
    assert st.snr == pytest.approx((1 - bm ** 16) ** 2 / (1 - bv ** 16), rel=1e-4)
    assert st.n_cos == 15 and st.steps == 16


@pytest.mark.parametrize("value", [0.37, 3.1e-5, 1e-21])
def test_uniform_gradient_is_isotropic_rank_one_and_undistorted(env, value):
    """Every coordinate sees the same gradient: v is constant, so A = 0 exactly and F (rank-one S) and C
    (constant preconditioner) vanish up to the absolute tolerance; 1e-21 puts v below the fp32 normal range."""
    torch, binding = env["torch"], env["binding"]
    blocks = [(0, 300 * 260, 300, 260), (78_016, 5_000), (83_072, 1030 * 3, 1030, 3), (86_208, 513 * 1027, 513, 1027)]
    n = 86_208 + 513 * 1027
    params = binding.default_profile_params()
    prof = binding.Profiler(blocks, params)
    orc = OracleRunner([W.BlockSpec(f"u{i}", b[1], *(b[2:] if len(b) > 2 else (0, 0)), offset=b[0]) for i, b in enumerate(blocks)],
                       None, **oracle_params(params))
    g = torch.full((n,), value, device="cuda:0")
    for _ in range(3):
        prof.step(g)
        orc.step_from_device(g)
    theta = 0.02 * torch.randn(n, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(3))
    stats, _ = prof.finalize(theta=theta)
    ostats, _ = orc.finalize([(1, 1, 0, 0, 32)], shapes=[(b[2], b[3]) if len(b) > 2 else (0, 0) for b in blocks], theta=theta)
    for i in range(len(blocks)):
        assert stats[i].A == 0.0 and stats[i].q10 == stats[i].q90
        assert abs(stats[i].F) <= 1e-6 and abs(stats[i].C) <= 1e-6, (i, stats[i].F, stats[i].C)
        assert_stats_close(stats[i], ostats[i], f"uniform {value} block {i}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("scale", [1e-22, 1e-19, 1e-12, 1e8])
def test_gradient_magnitudes_from_underflow_of_v_to_1e8(env, dtype, scale):
    """v-hat identically zero (1e-22), sub-normal (1e-19), tiny and huge: same statistics as the oracle."""
    w = ragged_workload(dtype, 1)
    for b in w.blocks:
        b.delta *= scale
        b.sigma *= scale
    run_both(env, w, 4, seed=77, theta_dtype=env["torch"].float32)


def test_three_thousand_small_blocks(env):
    """Blocks of 1..699 coordinates, some 7 x k and k x 2 matrices, tightly packed: one chunk and one
    histogram set per block."""
    rng = np.random.default_rng(5)
    blocks = []
    for i, n in enumerate(int(x) for x in rng.integers(1, 700, 3000)):
        r, c = (7, n // 7) if (n % 7 == 0 and n >= 14) else (0, 0)
        if n % 2 == 0 and i % 5 == 0:
            r, c = n // 2, 2
        blocks.append(W.BlockSpec(f"s{i}", n, r, c))
    w = W.Workload("many", blocks, 3, "bf16", "cycle", **W.K6)
    W.layout(w, 1); W.draw_stream_params(w, 9)
    run_both(env, w, 3, seed=5, theta_dtype=env["torch"].bfloat16)


def test_extreme_matrix_shapes(env):
    blocks = [W._mat("wide2", 2, 300001), W._mat("tall2", 300001, 2), W._mat("sq1k", 1000, 1000), W._mat("odd", 257, 255),
              W._mat("r1", 1, 5000), W._mat("c1", 5000, 1)]
    w = W.Workload("shapes", blocks, 3, "f32", "cycle", **W.K6)
    W.layout(w, 3); W.draw_stream_params(w, 4)
    run_both(env, w, 3, seed=6, theta_dtype=env["torch"].float32)


@pytest.mark.parametrize("kw", [dict(beta_m=0.5, beta_v=0.9, beta_rho=0.0), dict(eps=0.0), dict(eps=1e-3, eps_update=1e-2),
                                dict(beta_m=0.999, beta_v=0.99999)])
def test_profile_parameters_away_from_the_defaults(env, kw):
    run_both(env, ragged_workload("f32", 1), 4, **kw)


def test_caller_supplied_distortion_and_structure_residual(env):
    """C_raw / F_raw arrays take the place of the computed Eq. 6 / Eq. 7 values (also when theta is given);
    compute_F = False leaves F at 0."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload("f32", 64)
    params = binding.default_profile_params()
    prof = binding.Profiler(w.blocks, params)
    orc = OracleRunner(w.blocks, None, **oracle_params(params))
    buf = device.new_buffer(w)
    for t in range(1, 4):
        device.fill(w, buf, 21, t)
        prof.step(buf)
        orc.step_from_device(buf)
    n = len(w.blocks)
    rng = np.random.default_rng(3)
    C_raw, F_raw = rng.random(n) * 2.0, rng.random(n)
    theta = torch.randn(w.buffer_numel, device="cuda:0")
    stats, risk = prof.finalize(w.configs, C_raw=C_raw, F_raw=F_raw, theta=theta)
    rp = oracle.default_risk_params()
    for i in range(n):
        want = orc.state[i].finalize(rp, C_raw=float(C_raw[i]), F_raw=float(F_raw[i]))
        assert stats[i].C == C_raw[i] and stats[i].F == F_raw[i]
        assert_stats_close(stats[i], want, f"supplied C, F block {i}")
        assert_risk_close(risk[i], np.array([oracle.phi(want, c, False, rp) for c in w.configs]), f"block {i}")
    stats, _ = prof.finalize(w.configs, compute_F=False)
    assert all(stats[i].F == 0.0 and stats[i].s_F == 0.0 and stats[i].C == 0.0 for i in range(n))


def test_other_blocks_do_not_matter(env):
    torch, binding = env["torch"], env["binding"]
    blocks = [(0, 5000), (5003, 777), (6000, 30000)]
    g = [torch.randn(36000, device="cuda:0") for _ in range(3)]
    a = binding.Profiler(blocks); b = binding.Profiler([blocks[1]])
    for t in g:
        a.step(t)
        u = t.clone(); u[:5003] = 3.0; u[5780:] = -1.0
        b.step(u)
    sa, sb = a.finalize()[0][1], b.finalize()[0][0]
    assert bytes(sa) == bytes(sb)


def test_nan_gradient_poisons_only_its_block(env):
    torch, binding = env["torch"], env["binding"]
    blocks = [(0, 1000), (1024, 1000)]
    g = torch.randn(2048, device="cuda:0"); g[5] = float("nan")
    a = binding.Profiler(blocks)
    a.step(g); a.step(g)
    s = a.finalize()[0]
    assert np.isnan(s[0].m_sq) and np.isfinite(s[1].m_sq) and np.isfinite(s[1].lQ8) and s[1].rho_bar == pytest.approx(1.0)
    o = oracle.Block(1000); h = to_host_bits(g[:1000]); o.step(h); o.step(h)
    assert_stats_close(s[0], o.finalize(), "nan block")


def test_infinite_gradients_poison_only_their_block(env):
    """+inf and -inf coordinates in one block: its sums come out infinite or NaN exactly as in the oracle (NaN
    cosines and NaN Q count as 0), the quantiles still rank the finite second moments, the other block is untouched."""
    torch, binding = env["torch"], env["binding"]
    blocks = [(0, 1000), (1024, 1000)]
    clean = torch.randn(2048, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(5))
    g = clean.clone(); g[5] = float("inf"); g[300] = float("-inf")
    a, ref = binding.Profiler(blocks), binding.Profiler(blocks)
    for _ in range(2):
        a.step(g); ref.step(clean)
    s, r = a.finalize()[0], ref.finalize()[0]
    assert np.isinf(s[0].m_sq) and np.isinf(s[0].v_l1) and np.isfinite(s[0].q90) and np.isfinite(s[0].A)
    assert bytes(s[1]) == bytes(r[1])                      # the neighbour does not notice
    o = oracle.Block(1000); h = to_host_bits(g[:1000]); o.step(h); o.step(h)
    assert_stats_close(s[0], o.finalize(), "inf block")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_window_of_a_single_step(env, dtype):
    """finalize after the first step: the statistics come from the launch that does not read the states
    (no cosine yet, rho_bar = 0), F and C from v after one step."""
    torch = env["torch"]
    prof, stats, risk, ostats, orisk = run_both(env, ragged_workload(dtype, 1), 1,
                                                theta_dtype=torch.float32 if dtype == "f32" else torch.bfloat16)
    assert all(st.steps == 1 and st.n_cos == 0 and st.rho_bar == 0.0 for st in stats)


@pytest.mark.parametrize("seed", [2, 3])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_blocks_other_seeds(env, dtype, seed):
    """The ragged layout on the streams of seeds 2 and 3 (stream parameters and noise both drawn from the seed)."""
    torch = env["torch"]
    w = ragged_workload(dtype, 1)
    W.draw_stream_params(w, seed)
    run_both(env, w, 5, seed=seed, theta_dtype=torch.float32 if dtype == "f32" else torch.bfloat16)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mostly_dead_coordinates_overflow_the_candidate_lists(env, dtype):
    """60 % of the coordinates never see a gradient (v = 0 exactly), so the 0.1 quantile sits in a bin that
    holds most of every tile: the candidate lists of the matrix blocks overflow and their last digit comes from
    the third scan of v, while the block next to them (no dead coordinates) stays on its lists."""
    torch, binding = env["torch"], env["binding"]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    blocks = [W._mat("dead", 600, 520), W._vec("vec", 5000), W._mat("alive", 300, 260), W._mat("thin", 1030, 3)]
    w = W.Workload("dead", blocks, 3, dtype, "cycle", **W.K6)
    W.layout(w, 64)
    params = binding.default_profile_params(grad_dtype=0 if dtype == "f32" else 1)
    prof = binding.Profiler(w.blocks, params)
    orc = OracleRunner(w.blocks, None, **oracle_params(params))
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(99)
    dead = torch.rand(w.buffer_numel, device="cuda:0", generator=gen) < 0.6
    lo, hi = w.blocks[2].offset, w.blocks[2].offset + w.blocks[2].numel
    dead[lo:hi] = False
    for _ in range(3):
        g = torch.randn(w.buffer_numel, device="cuda:0", generator=gen) * 1e-3
        g[dead] = 0.0
        g = g.to(tdt)
        prof.step(g); orc.step_from_device(g)
    theta = (0.02 * torch.randn(w.buffer_numel, device="cuda:0", generator=gen)).to(tdt)
    stats, risk = prof.finalize(w.configs, theta=theta)
    ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in w.blocks], theta=theta)
    assert stats[0].q10 == 0.0 and stats[2].q10 > 0.0
    for i in range(len(w.blocks)):
        assert_stats_close(stats[i], ostats[i], f"dead block {i}")
    assert_risk_close(risk, orisk, "dead")


def test_captured_step_replays_as_later_steps(env):
    """A HIP graph captured from a steady-state step is replayed for the following steps (the step count lives on
    the device): same bits as eager steps on the same gradients, checked after every replay, with eager work and
    synchronisations between the replays."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload("bf16", 64)
    params = binding.default_profile_params(grad_dtype=1)
    grads = [device.fill(w, device.new_buffer(w), 41, t).clone() for t in range(1, 8)]
    prof, ref = binding.Profiler(w.blocks, params), binding.Profiler(w.blocks, params)
    gbuf = torch.zeros_like(grads[0])                      # the buffer the captured launch reads
    for t in (0, 1):
        gbuf.copy_(grads[t]); prof.step(gbuf); ref.step(grads[t])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        prof.step(gbuf)                                    # captured, not run
    for t in range(2, 7):
        gbuf.copy_(grads[t])
        graph.replay()
        ref.step(grads[t])                                 # eager work between the replays
        torch.cuda.synchronize()
        a, b = prof.finalize(w.configs)[0], ref.finalize(w.configs)[0]
        assert bytes(a) == bytes(b), f"after replay for step {t + 1}"
        assert a[0].steps == t + 1 and a[0].n_cos == t
    orc = OracleRunner(w.blocks, None, **oracle_params(params))
    for g in grads:
        orc.step_from_device(g)
    stats, risk = prof.finalize(w.configs)
    ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in w.blocks])
    for i in range(len(w.blocks)):
        assert_stats_close(stats[i], ostats[i], f"graph block {i}")
    assert_risk_close(risk, orisk, "graph")


def test_error_paths(env):
    torch, binding = env["torch"], env["binding"]
    prof = binding.Profiler([(0, 100), (200, 50)])
    with pytest.raises(binding.BaocError) as e:
        prof.finalize()                                   # no step yet
    assert e.value.status == binding.ERR_STATE
    g = torch.zeros(240, device="cuda:0")
    with pytest.raises(binding.BaocError) as e:
        prof.step(g)                                      # last block reaches element 250
    assert e.value.status == binding.ERR_INVALID
    prof.step(torch.zeros(250, device="cuda:0"))
    with pytest.raises(binding.BaocError) as e:
        prof.finalize([(1, 1, 0, 0, 4)])
    assert e.value.status == binding.ERR_INVALID
    with pytest.raises(TypeError):
        prof.step(torch.zeros(250, device="cuda:0", dtype=torch.bfloat16))
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    import ctypes as C
    h = C.c_void_p()
    arr = binding._block_array([(0, 100000)])
    p = binding.default_profile_params()
    assert binding.load_library().baoc_profile_begin(arr, 1, C.byref(p), ws.data_ptr(), 1024, C.byref(h)) == binding.ERR_WORKSPACE
    assert binding.load_library().baoc_profile_begin(arr, 1, C.byref(p), ws.data_ptr() + 1, 10 ** 9, C.byref(h)) == binding.ERR_WORKSPACE
