"""baoc_profile_begin_static: the profiler on the library's own per-GPU workspace array (no device allocation),
against baoc_profile_begin on a caller workspace, through the C ABI.  Needs an MI355X."""
import numpy as np
import pytest

from oracle.runner import OracleRunner, assert_risk_close, assert_stats_close, oracle_params
from synth import workloads as W
from test_gpu_parity import env  # noqa: F401

pytestmark = pytest.mark.gpu


def window(env, w, params, bufs, theta, workspace):
    """begin / one step per buffer / finalize / end on the given kind of workspace -> (stats as dicts, risk).
    Allocates nothing through torch when workspace == "static"."""
    torch, binding = env["torch"], env["binding"]
    prof = binding.Profiler(w.blocks, params, workspace=workspace)
    for b in bufs:
        prof.step(b)
    stats, risk = prof.finalize(w.configs, theta=theta)
    torch.cuda.synchronize()
    prof.close()
    return [s.asdict() for s in stats], risk


def same_bits(a, b):
    return all((x == y) or (np.isnan(x) and np.isnan(y)) for x, y in zip(a.values(), b.values()))


def test_static_workspace_matches_caller_workspace_twice_in_a_row(env):
    torch, binding, device = env["torch"], env["binding"], env["device"]
    big = W.make("gpt2_small")                       # does not fit the static array
    with pytest.raises(binding.BaocError) as e:
        binding.Profiler(big.blocks, binding.default_profile_params(), workspace="static")
    assert e.value.status == binding.ERR_WORKSPACE

    # first call: the ragged layout with bf16 gradients; second call: a smaller layout (fp32), on the array as the
    # first one left it
    cases = [(W.ragged("bf16", 3), 5, 11), (W.make("tiny"), 4, 12)]
    for w, T, seed in cases:
        bufs = []
        for t in range(1, T + 1):
            b = device.new_buffer(w); device.fill(w, b, seed, t); bufs.append(b)
        params = binding.default_profile_params(grad_dtype=1 if w.grad_dtype == "bf16" else 0)
        gen = torch.Generator(device="cuda:0"); gen.manual_seed(77)
        theta = 0.02 * torch.randn(w.buffer_numel, device="cuda:0", generator=gen)
        ref_stats, ref_risk = window(env, w, params, bufs, theta, None)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        got_stats, got_risk = window(env, w, params, bufs, theta, "static")
        assert torch.cuda.mem_get_info()[0] >= free_before          # nothing was taken from the device in between
        for i, (g, r) in enumerate(zip(got_stats, ref_stats)):
            assert same_bits(g, r), (w.name, i, g, r)               # same kernels, same order of sums: identical
        assert np.array_equal(got_risk, ref_risk)
        # and against the oracle, to the tolerance of every other parity test
        orc = OracleRunner(w.blocks, None, **oracle_params(params))
        for b in bufs:
            orc.step_from_device(b)
        ostats, orisk = orc.finalize(w.configs, shapes=[(b.rows, b.cols) for b in w.blocks], theta=theta)
        prof = binding.Profiler(w.blocks, params, workspace="static")
        for b in bufs:
            prof.step(b)
        stats, risk = prof.finalize(w.configs, theta=theta)
        for i in range(len(w.blocks)):
            assert_stats_close(stats[i], ostats[i], f"{w.name} block {i}")
        assert_risk_close(risk, orisk)
        # only one handle at a time may live on the array
        with pytest.raises(binding.BaocError) as e:
            binding.Profiler(w.blocks, params, workspace="static")
        assert e.value.status == binding.ERR_STATE
        prof.close()
