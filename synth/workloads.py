"""Seeded synthetic workloads: block layouts, per-block stream parameters and
allocation instances.  Input recipes only -- none of the profiler's or the
solver's arithmetic lives here.  Both the HIP path and the CPU oracle are fed
from this module; neither imports the other.

The layouts stand in for the vision / language / diffusion models of the
paper's experiments (Sec. 4.1), whose weights and datasets are not available:
only the tensor shapes matter to the profiler.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

# noise kinds of the gradient stream
GAUSS, STUDENT_T3 = 0, 1


@dataclass
class BlockSpec:
    name: str
    numel: int
    rows: int = 0          # rows*cols == numel for matrix blocks, else 0, 0
    cols: int = 0
    noise: int = GAUSS
    offset: int = 0        # elements from the start of the flat buffer (set by layout())
    # stream parameters (set by draw_stream_params())
    delta: float = 0.0     # strength of the persistent direction, U[0,1]
    sigma: float = 0.0     # noise level, log-uniform in [1e-4, 1e-1]
    s: float = 0.0         # log-normal spread of the per-coordinate scale kappa


@dataclass
class Workload:
    name: str
    blocks: List[BlockSpec]
    T: int                 # sampled steps in the window
    grad_dtype: str        # "f32" | "bf16"
    s_rule: str            # "cycle" ({0, .5, 2} round robin) | "uniform03"
    configs: List[tuple] = field(default_factory=list)   # (y_a, y_m, y_d, y_f, bits)
    config_names: List[str] = field(default_factory=list)
    time_cost: List[float] = field(default_factory=list)  # placeholder r_c per configuration
    mem_ratio: float = 0.5        # B_mem as a fraction of all-fp32-Adam state (8 B / element)
    time_cap_mean: Optional[float] = None   # B_time on the mean of r; None = slack
    buffer_numel: int = 0

    @property
    def numel(self):
        return sum(b.numel for b in self.blocks)


def _mat(name, rows, cols, **kw):
    return BlockSpec(name, rows * cols, rows, cols, **kw)


def _vec(name, n, **kw):
    return BlockSpec(name, n, 0, 0, **kw)


# ----------------------------------------------------------------------------
# layouts
# ----------------------------------------------------------------------------

def tiny_blocks():
    return [_mat(f"b{i}", 64, 64) for i in range(8)]


def resnet50_blocks():
    """Bottleneck residual network, stages [3,4,6,3], widths 64..512, x4 expansion,
    7x7 stem, 1000-way head: 53 convolutions, 53 x 2 norm vectors, FC weight + bias."""
    out = []

    def conv(name, cin, cout, k):
        out.append(_mat(name + ".w", cout, cin * k * k))
        out.append(_vec(name + ".bn.w", cout))
        out.append(_vec(name + ".bn.b", cout))

    conv("stem", 3, 64, 7)
    cin = 64
    for si, (n, w) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512])):
        for bi in range(n):
            p = f"s{si}.u{bi}"
            conv(p + ".c1", cin, w, 1)
            conv(p + ".c2", w, w, 3)
            conv(p + ".c3", w, 4 * w, 1)
            if bi == 0:
                conv(p + ".down", cin, 4 * w, 1)
            cin = 4 * w
    out.append(_mat("fc.w", 1000, 2048))
    out.append(_vec("fc.b", 1000))
    return out


def gpt2_blocks(n_layer, d, vocab, n_pos, heavy_tail_embeddings=True):
    """Decoder with learned positions, tied embedding, biased linears, two LN per layer."""
    out = []
    emb_noise = STUDENT_T3 if heavy_tail_embeddings else GAUSS
    out.append(_mat("wte", vocab, d, noise=emb_noise))
    out.append(_mat("wpe", n_pos, d, noise=emb_noise))
    for l in range(n_layer):
        p = f"h{l}"
        out += [_vec(p + ".ln1.w", d), _vec(p + ".ln1.b", d),
                _mat(p + ".qkv.w", d, 3 * d), _vec(p + ".qkv.b", 3 * d),
                _mat(p + ".proj.w", d, d), _vec(p + ".proj.b", d),
                _vec(p + ".ln2.w", d), _vec(p + ".ln2.b", d),
                _mat(p + ".fc.w", d, 4 * d), _vec(p + ".fc.b", 4 * d),
                _mat(p + ".fc2.w", 4 * d, d), _vec(p + ".fc2.b", d)]
    out += [_vec("lnf.w", d), _vec("lnf.b", d)]
    return out


def llama_blocks(n_layer=32, d=4096, ffn=11008, vocab=32000):
    out = [_mat("embed", vocab, d)]
    for l in range(n_layer):
        p = f"l{l}"
        out += [_vec(p + ".norm1", d),
                _mat(p + ".q", d, d), _mat(p + ".k", d, d), _mat(p + ".v", d, d), _mat(p + ".o", d, d),
                _vec(p + ".norm2", d),
                _mat(p + ".gate", ffn, d), _mat(p + ".up", ffn, d), _mat(p + ".down", d, ffn)]
    out += [_vec("norm_f", d), _mat("head", vocab, d)]
    return out


def unet_blocks(ctx=768, temb=1280, widths=(320, 640, 1280, 1280)):
    """Latent-diffusion style U-Net: residual units with time-embedding projections,
    transformer units (self + cross attention, gated MLP) on the three upper levels and
    in the middle, 3x3 down/up-sampling convolutions."""
    out = []

    def lin(name, cin, cout, bias=True):
        out.append(_mat(name + ".w", cout, cin))
        if bias:
            out.append(_vec(name + ".b", cout))

    def conv(name, cin, cout, k):
        out.append(_mat(name + ".w", cout, cin * k * k))
        out.append(_vec(name + ".b", cout))

    def norm(name, c):
        out.append(_vec(name + ".w", c))
        out.append(_vec(name + ".b", c))

    def res(name, cin, cout):
        norm(name + ".n1", cin); conv(name + ".c1", cin, cout, 3)
        lin(name + ".temb", temb, cout)
        norm(name + ".n2", cout); conv(name + ".c2", cout, cout, 3)
        if cin != cout:
            conv(name + ".skip", cin, cout, 1)

    def xf(name, c):
        norm(name + ".n", c); conv(name + ".in", c, c, 1)
        norm(name + ".ln1", c)
        for t in "qkv":
            lin(f"{name}.a1.{t}", c, c, bias=False)
        lin(name + ".a1.o", c, c)
        norm(name + ".ln2", c)
        lin(name + ".a2.q", c, c, bias=False)
        lin(name + ".a2.k", ctx, c, bias=False)
        lin(name + ".a2.v", ctx, c, bias=False)
        lin(name + ".a2.o", c, c)
        norm(name + ".ln3", c)
        lin(name + ".ff.in", c, 8 * c)
        lin(name + ".ff.out", 4 * c, c)
        conv(name + ".out", c, c, 1)

    lin("time.l1", widths[0], temb); lin("time.l2", temb, temb)
    conv("conv_in", 4, widths[0], 3)
    skips = [widths[0]]
    c = widths[0]
    for lv, w in enumerate(widths):
        for u in range(2):
            res(f"d{lv}.r{u}", c, w); c = w
            if lv < 3:
                xf(f"d{lv}.t{u}", w)
            skips.append(c)
        if lv < 3:
            conv(f"d{lv}.down", c, c, 3); skips.append(c)
    res("mid.r0", c, c); xf("mid.t", c); res("mid.r1", c, c)
    for lv in (3, 2, 1, 0):
        w = widths[lv]
        for u in range(3):
            res(f"u{lv}.r{u}", c + skips.pop(), w); c = w
            if lv < 3:
                xf(f"u{lv}.t{u}", w)
        if lv > 0:
            conv(f"u{lv}.up", c, c, 3)
    norm("out.n", c); conv("conv_out", c, 4, 3)
    return out


# ----------------------------------------------------------------------------
# candidate configurations (Def. 3.1) and their placeholder time costs
# ----------------------------------------------------------------------------

ADAM32, ADAM16, ADAM8 = (1, 1, 0, 0, 32), (1, 1, 0, 0, 16), (1, 1, 0, 0, 8)
SGDM32, SGD32, FACTORED32 = (0, 1, 0, 0, 32), (0, 0, 0, 0, 32), (1, 0, 0, 1, 32)

K4 = dict(configs=[ADAM32, ADAM8, ADAM16, SGD32],
          config_names=["adam32", "adam8", "adam16", "sgd32"],
          time_cost=[1.0, 1.3, 1.0, 0.4])
K6 = dict(configs=[ADAM32, ADAM16, ADAM8, SGDM32, SGD32, FACTORED32],
          config_names=["adam32", "adam16", "adam8", "sgdm32", "sgd32", "factored32"],
          time_cost=[1.0, 1.0, 1.3, 0.6, 0.4, 1.5])

MECHANISMS = {  # the seven mechanisms named in Sec. 4.1, as (y_a, y_m, y_d, y_f)
    "adamw": (1, 1, 1, 0), "adam": (1, 1, 0, 0), "sgd": (0, 0, 0, 0), "sgdm": (0, 1, 0, 0),
    "sgdw": (0, 0, 1, 0), "sgdwm": (0, 1, 1, 0), "adafactor": (1, 0, 0, 1)}


def k21():
    """The 7 mechanisms x {32,16,8} bits of Sec. 4.1."""
    cfgs, names, tc = [], [], []
    base_t = {"adamw": 1.0, "adam": 1.0, "sgd": 0.4, "sgdm": 0.6, "sgdw": 0.45, "sgdwm": 0.65, "adafactor": 1.5}
    for n, y in MECHANISMS.items():
        for b in (32, 16, 8):
            cfgs.append((*y, b)); names.append(f"{n}{b}")
            tc.append(base_t[n] * (1.3 if b == 8 else 1.0))
    return dict(configs=cfgs, config_names=names, time_cost=tc)


def make(name: str, pad: int = 64, seed: int = 1) -> Workload:
    if name == "tiny":
        w = Workload("tiny", tiny_blocks(), 16, "f32", "cycle", mem_ratio=0.5, **K4)
    elif name == "resnet50":
        w = Workload("resnet50", resnet50_blocks(), 32, "f32", "cycle", **K6)
    elif name == "gpt2_small":
        w = Workload("gpt2_small", gpt2_blocks(12, 768, 50257, 1024), 64, "f32", "cycle", **K6)
    elif name == "unet":
        w = Workload("unet", unet_blocks(), 32, "f32", "uniform03", **K6)
    elif name == "gpt_1p3b":
        w = Workload("gpt_1p3b", gpt2_blocks(24, 2048, 50257, 2048), 16, "f32", "cycle", **K6)
    elif name == "llama7b":
        w = Workload("llama7b", llama_blocks(), 16, "bf16", "cycle", mem_ratio=0.3,
                     time_cap_mean=1.3, **K6)
    else:
        raise KeyError(name)
    layout(w, pad)
    draw_stream_params(w, seed)
    return w


def ragged(dtype, pad, reverse=False):
    """Correctness layout: block sizes around the 64 / 256 / 1024 boundaries, 1- and 3-coordinate blocks,
    thin and ragged matrix shapes, optionally packed tightly (pad = 1: arbitrary offsets) or listed in
    reverse order.  K = 6 candidates, stream parameters of seed 5."""
    sizes = [1, 3, 63, 64, 255, 256, 257, 1000, 4099, 9408, 70001, 5, 1024 * 33 + 7]
    shapes = {3: (8, 8), 4: (5, 51), 5: (256, 1), 7: (10, 100), 8: (4099, 1), 9: (64, 147), 10: (70001, 1), 12: (73, 463)}
    blocks = []
    for i, n in enumerate(sizes):
        r, c = shapes.get(i, (0, 0))
        if r * c != n:
            r, c = (0, 0)
        blocks.append(BlockSpec(f"r{i}", n, r, c))
    blocks.append(_mat("wide", 3, 1027)); blocks.append(_mat("tall", 1030, 3)); blocks.append(_mat("sq", 300, 260))
    w = Workload("ragged", blocks, 5, dtype, "cycle", **K6)
    layout(w, pad); draw_stream_params(w, 5)
    if reverse:
        w.blocks.reverse()
    return w


WORKLOADS = ["tiny", "resnet50", "gpt2_small", "unet", "gpt_1p3b", "llama7b"]


def layout(w: Workload, pad: int = 64):
    """Place blocks back to back, each start rounded up to a multiple of `pad`
    elements (pad=1: tight packing, arbitrary offsets)."""
    off = 0
    for b in w.blocks:
        off = -(-off // pad) * pad
        b.offset = off
        off += b.numel
    w.buffer_numel = -(-off // 64) * 64


def draw_stream_params(w: Workload, seed: int = 1):
    rng = np.random.default_rng([seed, 0xBA0C])
    cyc = (0.0, 0.5, 2.0)
    for i, b in enumerate(w.blocks):
        b.delta = float(rng.uniform(0.0, 1.0))
        b.sigma = float(10.0 ** rng.uniform(-4.0, -1.0))
        b.s = cyc[i % 3] if w.s_rule == "cycle" else float(rng.uniform(0.0, 3.0))


# ----------------------------------------------------------------------------
# allocation instance (inputs of Eq. 2 other than the risk table)
# ----------------------------------------------------------------------------

def state_bytes(b: BlockSpec, cfg, qb: int = 256) -> int:
    """Persistent optimizer-state bytes M_{i,c} (StateMem restricted to a block):
    one state tensor per enabled mechanism, b/8 bytes per element, one fp32 absmax
    per group of qb elements for 8-bit states; a factored second moment keeps one
    row and one column vector for matrix blocks."""
    y_a, y_m, _y_d, y_f, bits = cfg

    def tensor(n):
        return n * (bits // 8) + (4 * (-(-n // qb)) if bits == 8 else 0)

    total = 0
    if y_m:
        total += tensor(b.numel)
    if y_a:
        if y_f and b.rows:
            total += tensor(b.rows) + tensor(b.cols)
        else:
            total += tensor(b.numel)
    return total


def allocation_inputs(w: Workload, qb: int = 256):
    """-> mem[N,K] int64 bytes, time[N,K] float64, B_mem bytes, time cap on the SUM of r."""
    N, K = len(w.blocks), len(w.configs)
    mem = np.zeros((N, K), np.int64)
    for i, b in enumerate(w.blocks):
        for k, c in enumerate(w.configs):
            mem[i, k] = state_bytes(b, c, qb)
    time = np.tile(np.asarray(w.time_cost, np.float64), (N, 1))
    b_mem = int(w.mem_ratio * 8 * w.numel)
    cap = float(w.time_cap_mean * N) if w.time_cap_mean is not None else float("inf")
    return mem, time, b_mem, cap
