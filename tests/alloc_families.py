"""Allocation instances at the sizes of the workloads: real per-block state bytes, the placeholder time costs, and
families of risk tables from continuous to tie-heavy.  Instance recipes only (inputs of Eq. 2); shared by the host
tests of baoc_allocate and of the oracle's solvers."""
import numpy as np

from synth import workloads as W

LAYOUTS = ["resnet50", "llama7b", "gpt_1p3b", "unet"]            # 161, 291, 292, 686 blocks
KINDS = ["continuous", "integer", "zero", "round1", "round3", "signals", "saturated",
         "continuous+", "integer+", "round1+", "round3+"]


def costs(name, K):
    """-> workload, candidate tuples, mem[N,K] bytes, time[N,K], memory budget, time cap 1.3 N on the sum."""
    w = W.make(name)
    cand = W.K6 if K == 6 else W.k21()
    cfgs, tcs = cand["configs"], cand["time_cost"]
    N = len(w.blocks)
    mem = np.array([[W.state_bytes(b, c) for c in cfgs] for b in w.blocks], np.int64)
    tc = np.tile(np.asarray(tcs, float), (N, 1))
    return w, cfgs, mem, tc, int(w.mem_ratio * 8 * w.numel), 1.3 * N


def signal_risk(rng, N, cfgs, levels=None, gamma=0.1):
    """Phi assembled like Eq. 9 + Eq. 1 from per-block signals; levels=None: continuous signals, otherwise every
    signal takes one of the given values (saturated signals: equal entries across blocks are the normal case)."""
    def draw():
        return rng.random(N) if levels is None else rng.choice(levels, N)
    sA, sM, sF = draw(), draw(), draw()
    Ct = rng.random(N) * 0.3 if levels is None else np.zeros(N)
    lQ = {32: np.zeros(N), 16: rng.random(N) * 1e-5 if levels is None else np.zeros(N),
          8: rng.random(N) * 0.5 if levels is None else rng.choice([0.0, 0.5], N)}
    risk = np.zeros((N, len(cfgs)))
    for k, (ya, ym, yd, yf, b) in enumerate(cfgs):
        agg = (1 - ya) + (1 - ym) + (1 - yd) + yf + 32.0 / b - 1
        risk[:, k] = sA * (1 - ya) + sM * (1 - ym) + Ct * (1 - yd) + sF * yf + lQ[b] + gamma * agg
    return risk


def family(rng, kind, N, cfgs, mem):
    K = len(cfgs)
    if kind.endswith("+"):                       # risk falls with the memory a configuration keeps: the budget binds
        r = 2.0 * (1.0 - mem / np.maximum(1, mem.max(1, keepdims=True))) + rng.random((N, K))
        return {"continuous+": r, "integer+": np.round(2 * r), "round1+": np.round(r, 1), "round3+": np.round(r, 3)}[kind]
    trend = rng.random((N, K)) * 2 + np.linspace(0, 1, K)[None, ::-1]
    if kind == "continuous":
        return trend
    if kind == "integer":
        return rng.integers(0, 5, (N, K)).astype(float)
    if kind == "zero":
        return np.zeros((N, K))
    if kind == "round1":
        return np.round(trend, 1)
    if kind == "round3":
        return np.round(trend, 3)
    if kind == "signals":
        return signal_risk(rng, N, cfgs)
    if kind == "saturated":
        return signal_risk(rng, N, cfgs, levels=[0.0, 0.5, 1.0])
    raise KeyError(kind)
