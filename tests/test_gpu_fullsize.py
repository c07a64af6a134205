"""Full-size layouts in the launch configuration the benchmark times; the oracle follows a sample
of blocks (every small block, the largest ones, a seeded 10 % draw).  The 7B-shaped layout runs its whole
window of 16 steps (about a minute of oracle time); the other windows are shortened.  Blocks are independent,
so a sampled block is checked exactly."""
import numpy as np
import pytest

from synth import workloads as W
from test_gpu_parity import check_allocation, env, run_both  # noqa: F401

pytestmark = pytest.mark.gpu


def sample_blocks(w, small=300_000, n_large=2, frac=0.1, cap=60_000_000, seed=11):
    """The n_large largest blocks, plus (smallest first, up to `cap` coordinates) every block of at
    most `small` coordinates and a seeded draw of `frac` of all blocks."""
    rng = np.random.default_rng(seed)
    order = np.argsort([-b.numel for b in w.blocks], kind="stable")
    large = [int(i) for i in order[:n_large]]
    rest = {i for i, b in enumerate(w.blocks) if b.numel <= small}
    rest |= {int(i) for i in rng.permutation(len(w.blocks))[:max(1, int(frac * len(w.blocks)))]}
    out, total = list(large), 0
    for i in sorted(rest - set(large), key=lambda i: (w.blocks[i].numel, i)):
        if total + w.blocks[i].numel <= cap:
            out.append(i); total += w.blocks[i].numel
    return sorted(out)


@pytest.mark.parametrize("name,T", [("unet", 6), ("gpt_1p3b", 4), ("llama7b", 16)])
def test_fullsize_sampled_blocks(env, name, T):  # noqa: F811
    w = W.make(name)
    only = sample_blocks(w)
    print(f"{name}: oracle follows {len(only)} of {len(w.blocks)} blocks, "
          f"{sum(w.blocks[i].numel for i in only):,} of {w.numel:,} coordinates, T={T}", flush=True)
    torch = env["torch"]
    prof, stats, risk, ostats, orisk = run_both(env, w, T, only=only, check_state=True,
                                                theta_dtype=torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32)
    check_allocation(env, w, risk)                      # the full risk table of the device run, all blocks


@pytest.mark.parametrize("seed", [2, 3])
def test_fullsize_unet_other_seeds(env, seed):  # noqa: F811
    """The UNet-shaped layout on the streams of seeds 2 and 3 (three seeds in all; seed 1 is the headline)."""
    w = W.make("unet", seed=seed)
    only = sample_blocks(w, seed=11 + seed)
    prof, stats, risk, ostats, orisk = run_both(env, w, 4, only=only, check_state=True, seed=seed, theta_dtype=env["torch"].float32)
    check_allocation(env, w, risk)


@pytest.mark.parametrize("name,seed", [("gpt_1p3b", 2), ("llama7b", 3)])
def test_fullsize_language_layouts_other_seeds(env, name, seed):  # noqa: F811
    """The 1.3B- and 7B-shaped layouts on another seed each (layout statistics and stream), short windows."""
    w = W.make(name, seed=seed)
    only = sample_blocks(w, seed=11 + seed, cap=40_000_000)
    torch = env["torch"]
    prof, stats, risk, ostats, orisk = run_both(env, w, 3, only=only, check_state=True, seed=seed,
                                                theta_dtype=torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32)
    check_allocation(env, w, risk)


def test_blocks_beyond_2_to_the_31_coordinates(env):  # noqa: F811
    """One vector block and one matrix block of more than 2^31 coordinates each, fed a constant gradient: the
    intensive statistics equal those of a small oracle block on the same gradient and the extensive ones scale
    with d exactly (no coordinate skipped or counted twice where 32-bit indices would wrap)."""
    import oracle
    from oracle.runner import oracle_params
    torch, binding = env["torch"], env["binding"]
    d_vec = (1 << 31) + (1 << 29) + 12_345
    rows, cols = 40_000, 60_001                                   # 2,400,040,000 > 2^31, cols not a multiple of 4
    off_mat = (d_vec + 63) // 64 * 64
    blocks = [(0, d_vec), (off_mat, rows * cols, rows, cols)]
    n = off_mat + rows * cols
    c = 0.375                                                     # exact in bf16
    params = binding.default_profile_params(grad_dtype=1)
    g = torch.full((n,), c, dtype=torch.bfloat16, device="cuda:0")
    theta = torch.full((n,), 0.5, dtype=torch.bfloat16, device="cuda:0")
    prof = binding.Profiler(blocks, params)
    small = oracle.Block(1000, **oracle_params(params))
    gs = np.full(1000, (np.float32(c).view(np.uint32) >> 16).astype(np.uint16), dtype=np.uint16)
    for _ in range(3):
        prof.step(g)
        small.step(gs)
    stats, _ = prof.finalize(theta=theta)
    want = small.finalize()
    for i, d in enumerate((d_vec, rows * cols)):
        st = stats[i]
        assert st.numel == d and st.steps == 3 and st.n_cos == 2
        assert st.A == 0.0 and st.q10 == want.q10 and st.q90 == want.q90
        assert abs(st.F) <= 1e-6 and abs(st.C) <= 1e-6
        for f in ("rho_bar", "snr", "Q16", "Q8", "err_m16", "err_v16", "err_m8", "err_v8"):
            assert getattr(st, f) == pytest.approx(getattr(want, f), rel=1e-5, abs=1e-7), f
        for f in ("m_sq", "v_l1", "g_sq_last"):
            assert getattr(st, f) == pytest.approx(getattr(want, f) * d / 1000.0, rel=1e-6), f
