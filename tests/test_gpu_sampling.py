"""Sparse coordinate sampling front end against the oracle (index sets and gathered values bit exact,
statistics of the sampled stream within the statistics tolerance)."""
import numpy as np
import pytest

import oracle
from oracle.runner import OracleRunner, assert_risk_close, assert_stats_close, oracle_params, to_host_bits
from synth import workloads as W
from test_gpu_parity import check_allocation, env, ragged_workload  # noqa: F401

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ratio", [0.001, 0.05, 1.0])
def test_index_sets_gather_and_sampled_statistics(env, dtype, ratio):  # noqa: F811
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = ragged_workload(dtype, 1)
    seed = 17
    smp = binding.Sampler(w.blocks, ratio, seed)
    idx, shapes = [], []
    for i, b in enumerate(w.blocks):
        want, shape = oracle.sample_indices_block(b.numel, b.rows, b.cols, ratio, seed, i)     # sub-matrix for matrix blocks
        want = want + np.uint64(b.offset)
        got = smp.indices(i).cpu().numpy().view(np.uint64)
        assert np.array_equal(got, want), f"Omega of block {i}"
        assert smp.compact_blocks[i][1] == want.size and tuple(smp.compact_blocks[i][2:]) == shape
        if shape == (0, 0):
            assert want.size == oracle.sample_count(b.numel, ratio)
        idx.append(want.astype(np.int64)); shapes.append(shape)
    assert any(sh != (0, 0) for sh in shapes) or ratio < 0.01
    params = binding.default_profile_params(grad_dtype=1 if dtype == "bf16" else 0)
    prof = binding.Profiler(smp.compact_blocks, params)
    orc = [oracle.Block(len(ix), **oracle_params(params)) for ix in idx]
    buf = device.new_buffer(w)
    compact = None
    for t in range(1, 5):
        device.fill(w, buf, 3, t)
        compact = smp.gather(buf, compact)
        host, chost = to_host_bits(buf), to_host_bits(compact)
        for i, ix in enumerate(idx):
            o, n = smp.compact_blocks[i][0], smp.compact_blocks[i][1]
            assert np.array_equal(chost[o:o + n], host[ix]), f"gathered values of block {i}"
            orc[i].step(host[ix])
        prof.step(compact)
    stats, _ = prof.finalize()
    for i in range(len(idx)):
        F = orc[i].structure_residual(*shapes[i])                    # Eq. 7 on the sampled sub-matrix
        assert_stats_close(stats[i], orc[i].finalize(F_raw=F), f"sampled block {i} ratio {ratio}")


def test_sampler_writes_stay_inside_its_buffers(env):  # noqa: F811
    torch, binding = env["torch"], env["binding"]
    w = ragged_workload("bf16", 1)
    blocks = [(b.offset, b.numel) for b in w.blocks]
    lib = binding.load_library()
    import ctypes as C
    arr = binding._block_array(blocks)
    compact = (binding.Block * len(blocks))()
    cn, wb = C.c_uint64(), C.c_uint64()
    assert lib.baoc_sample_layout(arr, len(blocks), 0.37, compact, C.byref(cn), C.byref(wb)) == 0
    band = 1 << 16
    arena = torch.full((band + wb.value + band,), 0x5A, dtype=torch.uint8, device="cuda:0")
    h = C.c_void_p()
    assert lib.baoc_sample_begin(arr, len(blocks), 0.37, 99, arena.data_ptr() + band, wb.value, C.byref(h)) == 0
    g = torch.randn(w.buffer_numel, device="cuda:0").to(torch.bfloat16)
    out = torch.full((cn.value + band,), 7.0, dtype=torch.bfloat16, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    assert lib.baoc_sample_gather(h, g.data_ptr(), g.numel(), binding.GRAD_BF16, out.data_ptr(), cn.value, st) == 0
    torch.cuda.synchronize()
    assert bool((arena[:band] == 0x5A).all()) and bool((arena[band + wb.value:] == 0x5A).all())
    assert bool((out[cn.value:] == 7.0).all())
    lib.baoc_sample_end(h)


def test_sampler_rejects_bad_arguments(env):  # noqa: F811
    torch, binding = env["torch"], env["binding"]
    for ratio in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(binding.BaocError) as e:
            binding.Sampler([(0, 100)], ratio)
        assert e.value.status == binding.ERR_INVALID
    smp = binding.Sampler([(0, 1000), (1000, 50)], 0.1)
    with pytest.raises(binding.BaocError) as e:
        smp.gather(torch.zeros(1049, device="cuda:0"))
    assert e.value.status == binding.ERR_INVALID
    with pytest.raises(binding.BaocError) as e:
        smp.gather(torch.zeros(1050, device="cuda:0"), torch.zeros(64, device="cuda:0"))
    assert e.value.status == binding.ERR_INVALID


def test_full_size_sampling_of_the_7b_layout(env):  # noqa: F811
    """s = 0.1 % of the 7B-shaped layout: index sets of sampled blocks bit exact, gather bit exact."""
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = W.make("llama7b")
    smp = binding.Sampler(w.blocks, 0.001, 5)
    buf = device.fill(w, device.new_buffer(w), 1, 1)
    compact = smp.gather(buf)
    torch.cuda.synchronize()
    for i in (0, 1, 2, 150, 289, 290):
        b = w.blocks[i]
        want, shape = oracle.sample_indices_block(b.numel, b.rows, b.cols, 0.001, 5, i)
        want = want.astype(np.int64) + b.offset
        assert np.array_equal(smp.indices(i).cpu().numpy(), want) and tuple(smp.compact_blocks[i][2:]) == shape
        o, n = smp.compact_blocks[i][0], smp.compact_blocks[i][1]
        assert torch.equal(compact[o:o + n], buf[torch.from_numpy(want).cuda()])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_full_size_sampled_window_of_the_7b_layout(env, seed):  # noqa: F811
    """The front end of Sec. 3.1 at its real shape and the paper's ratio: s = 0.1 % of the 7B-shaped layout (6.7 M of
    6.7 G coordinates), gradient streams of seeds 1 to 3.  Every gathered value is its sampled coordinate's; the
    profiler on the compact layout agrees with the oracle on every block (F of Eq. 7 on the sampled sub-matrices, C of
    Eq. 6 on the sampled parameters); the allocation for the full-size costs on that risk table is the oracle's."""
    from collections import namedtuple
    torch, binding, device = env["torch"], env["binding"], env["device"]
    w = W.make("llama7b", seed=seed)
    smp = binding.Sampler(w.blocks, 0.001, 5)
    CB = namedtuple("CB", "offset numel rows cols")
    cblocks = [CB(*b) for b in smp.compact_blocks]
    assert sum(b.rows > 0 for b in cblocks) == sum(b.rows > 0 for b in w.blocks)          # every matrix block keeps a matrix form
    params = binding.default_profile_params(grad_dtype=1)
    prof = binding.Profiler(smp.compact_blocks, params)
    orc = OracleRunner(cblocks, None, **oracle_params(params))
    idx = [smp.indices(i) for i in range(len(w.blocks))]
    buf, compact = device.new_buffer(w), None
    for t in range(1, 5):
        device.fill(w, buf, seed, t)
        compact = smp.gather(buf, compact)
        for i, b in enumerate(cblocks):
            assert torch.equal(compact[b.offset:b.offset + b.numel], buf[idx[i]]), f"gathered values of block {i}, step {t}"
        prof.step(compact)
        orc.step_from_device(compact)
    del buf
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(99 + seed)
    theta = torch.empty(w.buffer_numel, dtype=torch.bfloat16, device="cuda:0")
    for o in range(0, w.buffer_numel, 1 << 28):                                          # in pieces: no 27 GB fp32 temporary
        n = min(1 << 28, w.buffer_numel - o)
        theta[o:o + n] = (0.02 * torch.randn(n, device="cuda:0", generator=gen)).to(torch.bfloat16)
    ctheta = smp.gather(theta)
    stats, risk = prof.finalize(w.configs, theta=ctheta)
    ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in cblocks], theta=ctheta)
    for i, b in enumerate(cblocks):
        assert_stats_close(stats[i], ostats[i], f"sampled block {i} ({w.blocks[i].name}, {b.numel} of {w.blocks[i].numel})")
        assert_risk_close(risk[i], orisk[i], f"sampled block {i}")
    assert sum(st.F > 0 for st in stats) * 2 >= sum(b.rows > 1 and b.cols > 1 for b in cblocks) > 200        # F exists under sampling
    check_allocation(env, w, risk)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_device_gradient_generator_matches_its_host_twin(env, dtype):  # noqa: F811
    """Same counter-based stream on both sides: the device evaluates the transcendentals in
    float32, the twin in float64, so blocks agree in norm to ~1e-6 and nearly all bf16 codes match."""
    from synth import gradgen
    device = env["device"]
    w = ragged_workload(dtype, 64)
    w.blocks[2].noise = W.STUDENT_T3
    w.blocks[9].noise = W.STUDENT_T3
    got = to_host_bits(device.fill(w, device.new_buffer(w), 9, 4))
    want = gradgen.flat_gradient(w, 9, 4)
    if dtype == "bf16":
        assert np.mean(got == want) > 0.98
        got, want = gradgen.bf16_bits_to_f32(got), gradgen.bf16_bits_to_f32(want)
    got, want = got.astype(np.float64), want.astype(np.float64)
    tol = 2.0 ** -7 if dtype == "bf16" else 1e-5
    for i, b in enumerate(w.blocks):
        a, r = got[b.offset:b.offset + b.numel], want[b.offset:b.offset + b.numel]
        assert np.linalg.norm(a - r) <= tol * np.linalg.norm(r), f"block {i}"
        assert np.max(np.abs(a - r)) <= 10 * tol * np.max(np.abs(r)), f"block {i}"
    used = np.zeros(w.buffer_numel, bool)
    for b in w.blocks:
        used[b.offset:b.offset + b.numel] = True
    assert not got[~used].any()                                   # gaps between blocks stay zero


def test_pure_stream_of_the_benchmark_stays_in_bounds(env):  # noqa: F811
    """Harness check of the pure-stream kernel behind the benchmark's practical ceiling: it rewrites m, v, g_prev of
    exactly n coordinates and refuses sizes it cannot cover."""
    torch, device = env["torch"], env["device"]
    L = device.probe_lib()
    n, pad = 512 * 37, 4096
    m = torch.randn(n + pad, device="cuda:0"); v = torch.rand(n + pad, device="cuda:0")
    gp = torch.randn(n + pad, device="cuda:0").to(torch.bfloat16); g = torch.randn(n + pad, device="cuda:0").to(torch.bfloat16)
    m0, v0, gp0 = m.clone(), v.clone(), gp.clone()
    st = torch.cuda.current_stream().cuda_stream
    assert L.synth_mix_stream(n, m.data_ptr(), v.data_ptr(), gp.data_ptr(), g.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert torch.allclose(m[:n], m0[:n] * 0.9 + v0[:n], rtol=1e-6, atol=1e-6) and torch.allclose(v[:n], v0[:n] * 0.999 + m0[:n], rtol=1e-6, atol=1e-6)
    assert torch.equal(m[n:], m0[n:]) and torch.equal(v[n:], v0[n:]) and torch.equal(gp[n:], gp0[n:])
    assert not torch.equal(gp[:n], gp0[:n])
    assert L.synth_mix_stream(n + 1, m.data_ptr(), v.data_ptr(), gp.data_ptr(), g.data_ptr(), st) == -1
    assert L.synth_mix_stream(n, 0, v.data_ptr(), gp.data_ptr(), g.data_ptr(), st) == -1
