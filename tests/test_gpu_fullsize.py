"""Full-size layouts in the launch configuration the benchmark times; the oracle follows a sample
of blocks (every small block, the largest ones, a seeded 10 % draw).  The 7B-shaped layout runs its whole
window of 16 steps (about a minute of oracle time); the other windows are shortened.  Blocks are independent,
so a sampled block is checked exactly."""
import numpy as np
import pytest

from synth import workloads as W
from test_gpu_parity import env, run_both  # noqa: F401

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
    run_both(env, w, T, only=only, check_state=True,
             theta_dtype=torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32)
