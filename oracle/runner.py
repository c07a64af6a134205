"""Running the oracle next to a device stream and comparing results with it.

TEST INFRASTRUCTURE ONLY, like the rest of this package: used by the tests, by the smoke check and by the
benchmark's cpu_baseline leg.  Holds no arithmetic of the method: it copies device buffers to the host, feeds
them to oracle.Block and states the tolerance of the comparison."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle

RTOL, ATOL = 1e-4, 1e-6          # |gpu - oracle| <= 1e-6 + 1e-4 |oracle| for every reported statistic
INT_FIELDS = ("numel", "steps", "n_cos")
THREADS = 16


def to_host_bits(t):
    """torch tensor (fp32 or bf16, any device) -> numpy float32 or uint16 bit patterns."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def assert_stats_close(got, want, where=""):
    """got: BlockStats from the library, want: oracle.Stats."""
    for f in INT_FIELDS:
        assert getattr(got, f) == getattr(want, f), f"{where} {f}: {getattr(got, f)} != {getattr(want, f)}"
    for f in oracle.STAT_FIELDS:
        if f in INT_FIELDS:
            continue
        g, w = getattr(got, f), getattr(want, f)
        if np.isnan(w) or np.isnan(g):
            assert np.isnan(w) and np.isnan(g), f"{where} {f}: {g} vs {w}"
            continue
        if g == w:                                       # also equal infinities (after a non-finite gradient)
            continue
        assert abs(g - w) <= ATOL + RTOL * abs(w), f"{where} {f}: gpu {g!r} oracle {w!r} diff {abs(g - w):.3e}"


def assert_risk_close(got, want, where=""):
    got, want = np.asarray(got), np.asarray(want)
    bad = np.abs(got - want) > ATOL + RTOL * np.abs(want)
    assert not bad.any(), f"{where} risk entries differ at {np.argwhere(bad)[:5].tolist()}: {got[bad][:5]} vs {want[bad][:5]}"


class OracleRunner:
    """Oracle over a subset of blocks, threads over blocks (each block is sequential, as written)."""

    def __init__(self, blocks, only=None, **params):
        self.blocks = [(int(b.offset), int(b.numel)) for b in blocks]
        self.only = list(range(len(blocks))) if only is None else list(only)
        self.state = {i: oracle.Block(self.blocks[i][1], **params) for i in self.only}
        self.pool = ThreadPoolExecutor(THREADS)

    def step_from_device(self, buf):
        """Copies the sampled blocks' slices of the device buffer to the host and steps the oracle."""
        slices = {i: to_host_bits(buf[self.blocks[i][0]:self.blocks[i][0] + self.blocks[i][1]]) for i in self.only}
        list(self.pool.map(lambda i: self.state[i].step(slices[i]), self.only))

    def finalize(self, configs, rp=None, pref_mask=None, shapes=None, theta=None):
        """shapes: (rows, cols) per block -> F from Eq. 7; theta: flat device tensor -> C from Eq. 6."""
        rp = rp or oracle.default_risk_params()

        def one(i):
            F = self.state[i].structure_residual(*shapes[i]) if shapes is not None else 0.0
            C = 0.0
            if theta is not None:
                o, n = self.blocks[i]
                C = self.state[i].distortion(to_host_bits(theta[o:o + n]))
            return self.state[i].finalize(rp, C_raw=C, F_raw=F)
        stats = list(self.pool.map(one, self.only))
        risk = np.array([[oracle.phi(st, c, bool(pref_mask[k]) if pref_mask is not None else False, rp)
                          for k, c in enumerate(configs)] for st in stats])
        return dict(zip(self.only, stats)), risk


def oracle_params(p):
    """ProfileParams of the binding -> keyword arguments of oracle.Block."""
    return dict(beta_m=p.beta_m, beta_v=p.beta_v, beta_rho=p.beta_rho, eps=p.eps, eps_u=p.eps_update, qb=p.quant_block)
