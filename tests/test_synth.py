"""The synthetic workloads: layouts have the sizes the configs name, the stream has the stated moments."""
import numpy as np
import pytest

from synth import gradgen, workloads as W

EXPECT = {"tiny": (8, 32_768), "resnet50": (161, 25_557_032), "gpt2_small": (148, 124_439_808),
          "unet": (686, 859_520_964), "gpt_1p3b": (292, 1_315_723_264), "llama7b": (291, 6_738_415_616)}


@pytest.mark.parametrize("name", W.WORKLOADS)
def test_layout_sizes(name):
    w = W.make(name)
    assert (len(w.blocks), w.numel) == EXPECT[name]
    ends = 0
    for b in w.blocks:
        assert b.offset % 64 == 0 and b.offset >= ends and (b.rows * b.cols in (0, b.numel))
        ends = b.offset + b.numel
    assert w.buffer_numel >= ends
    tight = W.make(name, pad=1)
    assert tight.blocks[-1].offset + tight.blocks[-1].numel == tight.numel


def test_stream_parameters_follow_the_recipe():
    w = W.make("unet", seed=3)
    d = np.array([b.delta for b in w.blocks]); s = np.array([b.sigma for b in w.blocks]); k = np.array([b.s for b in w.blocks])
    assert 0 <= d.min() and d.max() <= 1 and 1e-4 <= s.min() and s.max() <= 1e-1 and 0 <= k.min() and k.max() <= 3
    assert [b.s for b in W.make("tiny").blocks[:4]] == [0.0, 0.5, 2.0, 0.0]
    assert W.make("gpt2_small").blocks[0].noise == W.STUDENT_T3 and W.make("gpt2_small").blocks[5].noise == W.GAUSS


def test_generator_moments_and_reproducibility():
    spec = W.BlockSpec("b", 200_000, delta=0.0, sigma=1.0, s=0.0)
    g = gradgen.block_gradient(1, 0, spec, 1).astype(np.float64)
    assert abs(g.mean()) < 0.01 and g.std() == pytest.approx(1.0, abs=0.01)
    assert np.array_equal(gradgen.block_gradient(1, 0, spec, 1), gradgen.block_gradient(1, 0, spec, 1))
    assert not np.array_equal(gradgen.block_gradient(1, 0, spec, 1), gradgen.block_gradient(1, 0, spec, 2))
    part = gradgen.block_gradient(1, 0, spec, 1, 1000, 1100)                  # any element on its own
    assert np.array_equal(part, gradgen.block_gradient(1, 0, spec, 1)[1000:1100])
    t = W.BlockSpec("t", 200_000, delta=0.0, sigma=1.0, s=0.0, noise=W.STUDENT_T3)
    h = gradgen.block_gradient(1, 0, t, 1).astype(np.float64)
    assert np.mean(np.abs(h) > 4) > 5 * np.mean(np.abs(g) > 4)                # heavier tails
    drift = W.BlockSpec("d", 100_000, delta=1.0, sigma=0.0, s=0.0)
    u = gradgen.block_gradient(1, 0, drift, 1).astype(np.float64)
    assert np.linalg.norm(u) == pytest.approx(1.0, abs=0.01)                  # the persistent direction has unit length


def test_bf16_packing_round_trip():
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    bits = gradgen.f32_to_bf16_bits(x)
    back = gradgen.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(gradgen.f32_to_bf16_bits(back), bits)


def test_state_bytes_model():
    b = W._mat("m", 100, 300)
    assert W.state_bytes(b, W.ADAM32) == 2 * 4 * 30000
    assert W.state_bytes(b, W.ADAM16) == 2 * 2 * 30000
    assert W.state_bytes(b, W.ADAM8) == 2 * (30000 + 4 * 118)                 # one fp32 absmax per 256 elements
    assert W.state_bytes(b, W.SGDM32) == 4 * 30000 and W.state_bytes(b, W.SGD32) == 0
    assert W.state_bytes(b, W.FACTORED32) == 4 * 400
    assert W.state_bytes(W._vec("v", 77), W.FACTORED32) == 4 * 77
    # the paper's own consistency datum: GPT2-small under AdamW16 is 475.15 MB (Table 3);
    # 2 states x 2 bytes x 124,439,808 parameters = 474.70 MiB
    w = W.make("gpt2_small")
    total = sum(W.state_bytes(b, (1, 1, 1, 0, 16)) for b in w.blocks)
    assert total / 2 ** 20 == pytest.approx(475.15, rel=2e-3)
