#!/usr/bin/env python3
"""Benchmark of the BAOC gradient-stream profiler on one MI355X.

A "step" of the contract is 1/K of one profiling window: the timed region holds
baoc_profile_begin, K calls of baoc_profile_step on gradients already resident in
HBM, baoc_profile_finalize (quantile selection, structure residual, distortion
against a resident parameter buffer, metrics, risk table) and baoc_allocate.  `value` = K * D / (time of that region) in gradient elements per
second.  The roofline object is about the dominant kernel alone (the fused step
pass), timed with HIP events on the launch stream inside the same region.

Prints ONE JSON line.  The CPU oracle appears only in the cpu_baseline leg.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
BYTES_PER_ELEM = {"f32": 28, "bf16": 22}   # g read, g_prev read+write, m and v read+write


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="K profile steps in the timed window (0 = the workload's T)")
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--ring", type=int, default=4, help="distinct pre-generated gradient buffers cycled through")
    ap.add_argument("--chunk-groups", type=int, default=0, help="launch shape of the step kernel, 0 = library default")
    ap.add_argument("--chunk-slices", type=int, default=0)
    ap.add_argument("--groups-per-wave", type=int, default=0)
    ap.add_argument("--waves-per-workgroup", type=int, default=0)
    ap.add_argument("--resident-workgroups", type=int, default=0)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB -> 1 GiB device copy (reference dispatch for rocprofv3 --pmc byte counters)")
    ap.add_argument("--sample-ratio", type=float, default=0.0,
                    help="sparse coordinate sampling (Sec. 3.1): gather g[Omega] with this ratio before every step and profile "
                         "the compact buffer; prints its own JSON line (not the headline metric)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the steady-state step figures of the gpt_1p3b and unet layouts and the pure-stream ceiling "
                         "that the default run appends to its line")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "k_step_pmc_traffic.txt"))
    return ap.parse_args()


def read_traffic(path, workload):
    """`<workload> traffic_bytes_per_launch <N>` lines written from rocprofv3 --pmc runs, or None."""
    try:
        for line in open(path):
            f = line.split("#", 1)[0].split()
            if len(f) >= 3 and f[0] == workload and f[1] == "traffic_bytes_per_launch":
                return float(f[2])
    except OSError:
        pass
    return None


def cpu_baseline(w, ring, seed, params):
    """The oracle as it stands, threads over blocks, on a bounded sample of the same workload."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from oracle.runner import oracle_params, to_host_bits
    budget = 250_000_000                                  # coordinates in the sample
    order = sorted(range(len(w.blocks)), key=lambda i: (abs(w.blocks[i].numel - 16_777_216), i))
    pick, tot = [], 0
    for i in order:
        if tot + w.blocks[i].numel <= budget and len(pick) < 16:
            pick.append(i); tot += w.blocks[i].numel
    if not pick:
        pick = [min(range(len(w.blocks)), key=lambda i: w.blocks[i].numel)]; tot = w.blocks[pick[0]].numel
    steps = min(w.T, 16)                                  # up to a whole window of the sample: about 10 s on 16 cores
    per_ring = [[to_host_bits(g[w.blocks[i].offset:w.blocks[i].offset + w.blocks[i].numel]) for i in pick] for g in ring]
    data = [per_ring[t % len(ring)] for t in range(steps)]
    blocks = [oracle.Block(w.blocks[i].numel, **oracle_params(params)) for i in pick]
    cores = min(16, os.cpu_count() or 1, len(pick))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as pool:
        for t in range(steps):
            list(pool.map(lambda k: blocks[k].step(data[t][k]), range(len(pick))))
        list(pool.map(lambda b: b.finalize(), blocks))
    dt = time.perf_counter() - t0
    # the same oracle on one core: the first sampled block alone, two steps + finalize
    one = oracle.Block(w.blocks[pick[0]].numel, **oracle_params(params))
    t1 = time.perf_counter()
    for t in range(2):
        one.step(data[t][0])
    one.finalize()
    dt1 = time.perf_counter() - t1
    return {"value": tot * steps / dt, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(pick)} blocks ({tot:,} coordinates) of {w.name}, {steps} steps + finalize, threads over blocks",
            "seconds": round(dt, 3),
            "one_core": {"value": w.blocks[pick[0]].numel * 2 / dt1, "unit": "elements/s",
                         "sample": f"1 block ({w.blocks[pick[0]].numel:,} coordinates), 2 steps + finalize", "seconds": round(dt1, 3)}}


def sampled_windows(a, w, ring, theta, params, mem, tc, b_mem, cap):
    """Window with the sparse-sampling front end: Omega drawn once, then per step one gather of g[Omega] into a
    compact buffer and one profiler step on it; theta is gathered the same way for Eq. 6."""
    import torch
    import paper_2605_04711_amd as B
    from paper_2605_04711_amd import binding
    K, D, R = a.steps or w.T, w.numel, len(ring)
    smp = binding.Sampler(w.blocks, a.sample_ratio, a.seed)
    samples = sum(b[1] for b in smp.compact_blocks)
    compact = torch.zeros(smp.compact_numel, dtype=ring[0].dtype, device=ring[0].device)
    theta_c = smp.gather(theta)
    esz = ring[0].element_size()

    def window(steps):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prof = binding.Profiler(smp.compact_blocks, params, device=ring[0].device)
        for t in range(steps):
            ev[t][0].record(); smp.gather(ring[t % R], compact)
            ev[t][1].record(); prof.step(compact)
            ev[t][2].record()
        stats, risk = prof.finalize(w.configs, theta=theta_c)
        t2 = time.perf_counter()
        B.allocate(risk, mem, tc, b_mem, cap)
        t3 = time.perf_counter()
        g_ms = [e[0].elapsed_time(e[1]) for e in ev]; s_ms = [e[1].elapsed_time(e[2]) for e in ev]
        prof.close()
        return t3 - t0, g_ms, s_ms, (t2 - t0) * 1e3 - sum(g_ms) - sum(s_ms)

    if a.warmup > 0:
        window(a.warmup)
    total, g_ms, s_ms, rest_ms = window(K)
    g_avg = sum(g_ms) / len(g_ms); s_avg = sum(s_ms[1:]) / max(1, len(s_ms) - 1)
    gather_bytes = samples * (8 + 2 * esz)                # index, element read, element written
    return {"metric": "gradient elements covered/sec with sparse sampling", "value": K * D / total, "unit": "elements/s",
            "n_gpus": 1, "steps": K, "warmup": a.warmup, "ms_per_step": total * 1e3 / K, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"{w.name} with sampling ratio {a.sample_ratio}: {samples:,} of {D:,} coordinates in Omega, "
                                   f"window of {K} x (gather + step) + finalize + allocate", "samples": samples},
            "breakdown_ms": {"gather_avg": round(g_avg, 4), "step_avg": round(s_avg, 4), "begin_finalize": round(rest_ms, 3)},
            "roofline": {"bound": "hbm", "kernel": "k_gather", "achieved": gather_bytes / (g_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": gather_bytes / (g_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                         "algorithmic_bytes_per_launch": gather_bytes, "avg_launch_ms": g_avg, "launches": len(g_ms)}}


def practical_ceiling(w, g, dev):
    """What this HBM system delivers for the step kernel's byte mix with no arithmetic: a pure stream of
    22 bytes per coordinate (4 reads, 3 writes) in its best launch shape, median of 5 launches.  bf16 gradients only."""
    import torch
    from synth import device
    if w.grad_dtype != "bf16":
        return None
    L = device.probe_lib()
    n = min(w.numel, g.numel()) // 512 * 512
    m = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros_like(m)
    gp = torch.zeros(n, dtype=torch.bfloat16, device=dev)
    st = torch.cuda.current_stream(dev).cuda_stream

    def launch():
        rc = L.synth_mix_stream(n, m.data_ptr(), v.data_ptr(), gp.data_ptr(), g.data_ptr(), st)
        if rc:
            raise RuntimeError(f"synth_mix_stream: {rc}")
    launch(); torch.cuda.synchronize()
    ms = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); launch(); e1.record(); e1.synchronize()
        ms.append(e0.elapsed_time(e1))
    t = sorted(ms)[2]
    gbs = 22 * n / t / 1e6
    return {"GB/s": gbs, "frac": gbs / HBM_PEAK_GBS, "ms": t, "coordinates": n,
            "what": "pure stream of the step kernel's 22 B/coordinate (4 reads, 3 writes, no arithmetic): single-wavefront "
                    "workgroups of 2 groups, 4 resident per CU; median of 5 launches"}


def secondary_steps(names, a, dev):
    """Steady-state step launches of further layouts (begin, the first step, then `launches` timed steps each)."""
    import torch
    from paper_2605_04711_amd import binding
    from synth import device, workloads as W
    out = []
    for name in names:
        w = W.make(name, seed=a.seed)
        params = binding.default_profile_params(grad_dtype=1 if w.grad_dtype == "bf16" else 0)
        ring = [device.fill(w, device.new_buffer(w, dev), a.seed, t + 1) for t in range(2)]
        prof = binding.Profiler(w.blocks, params, device=dev)
        launches = 8
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches + 2)]
        for t in range(launches + 2):                                   # launch 0: first-step kernel, launch 1: warm-up
            ev[t][0].record(); prof.step(ring[t % 2]); ev[t][1].record()
        torch.cuda.synchronize()
        ms = [e0.elapsed_time(e1) for e0, e1 in ev][2:]
        prof.close()
        del prof, ring
        avg = sum(ms) / len(ms)
        bpe = BYTES_PER_ELEM[w.grad_dtype]
        out.append({"workload": name, "blocks": len(w.blocks), "coordinates": w.numel, "grad_dtype": w.grad_dtype,
                    "kernel": "k_step (steady state)", "avg_launch_ms": avg, "min_launch_ms": min(ms), "launches": launches,
                    "algorithmic_bytes_per_launch": bpe * w.numel, "achieved": bpe * w.numel / avg / 1e6, "unit": "GB/s",
                    "frac": bpe * w.numel / avg / 1e6 / HBM_PEAK_GBS, "step_only_elements_per_s": w.numel / (avg * 1e-3)})
        torch.cuda.empty_cache()
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build profiles on ONE GPU (no sharding or collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2605_04711_amd as B
    from paper_2605_04711_amd import binding
    from synth import device, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load_library(); device.lib()
    dev = torch.device("cuda:0")
    w = W.make(a.workload, seed=a.seed)
    K = a.steps or w.T
    D = w.numel
    params = binding.default_profile_params(grad_dtype=1 if w.grad_dtype == "bf16" else 0, chunk_groups=a.chunk_groups,
                                            chunk_slices=a.chunk_slices, groups_per_wave=a.groups_per_wave,
                                            waves_per_workgroup=a.waves_per_workgroup, resident_workgroups=a.resident_workgroups)
    mem, tc, b_mem, cap = W.allocation_inputs(w)
    cap = 1e12 if not np.isfinite(cap) else cap

    # inputs resident in HBM before the clock starts
    R = max(1, min(a.ring, K))
    ring = [device.fill(w, device.new_buffer(w, dev), a.seed, t + 1) for t in range(R)]
    nbytes = binding.workspace_bytes(w.blocks, params)
    # parameters theta for the distortion metric (Eq. 6), same layout and dtype as the gradients
    gen = torch.Generator(device=dev); gen.manual_seed(a.seed)
    theta = torch.empty(w.buffer_numel, dtype=ring[0].dtype, device=dev)
    for lo in range(0, w.buffer_numel, 1 << 28):               # in slices: keeps the fp32 temporary small
        n = min(1 << 28, w.buffer_numel - lo)
        theta[lo:lo + n] = (0.02 * torch.randn(n, device=dev, generator=gen)).to(theta.dtype)
    torch.cuda.synchronize()

    def window(steps, timed):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prof = binding.Profiler(w.blocks, params, device=dev)            # baoc_profile_begin (workspace from torch)
        t1 = time.perf_counter()
        for t in range(steps):
            ev[t][0].record()
            prof.step(ring[t % R])
            ev[t][1].record()
        stats, risk = prof.finalize(w.configs, theta=theta)
        t2 = time.perf_counter()
        choice, obj, m_used, t_used = B.allocate(risk, mem, tc, b_mem, cap)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        step_ms = [e0.elapsed_time(e1) for e0, e1 in ev]
        prof.close()
        del prof
        return dict(total=t3 - t0, begin=t1 - t0, steps_and_finalize=t2 - t1, allocate=t3 - t2, step_ms=step_ms,
                    obj=obj, mem_used=m_used, choice=choice, stats=stats)

    if a.sample_ratio > 0:
        print(json.dumps(sampled_windows(a, w, ring, theta, params, mem, tc, b_mem, cap)))
        return
    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if a.warmup > 0:
        window(a.warmup, False)
    r = window(K, True)
    step_ms = r["step_ms"]
    # The first launch after begin is another kernel instantiation (states known to be zero, not
    # read: 12 or 16 B per coordinate); the roofline is about the steady-state kernel, launches 2..K.
    steady = step_ms[1:] if len(step_ms) > 1 else step_ms
    avg_ms = sum(steady) / len(steady)
    bpe = BYTES_PER_ELEM[w.grad_dtype]
    achieved = bpe * D / (avg_ms * 1e-3) / 1e9
    finalize_ms = r["steps_and_finalize"] * 1e3 - sum(step_ms)
    traffic = read_traffic(a.traffic_file, w.name)

    out = {
        "metric": "gradient elements profiled/sec",
        "value": K * D / r["total"],
        "unit": "elements/s",
        "n_gpus": 1, "steps": K, "warmup": a.warmup,
        "ms_per_step": r["total"] * 1e3 / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {len(w.blocks)} blocks, {D:,} coordinates, {w.grad_dtype} gradients, "
                               f"fp32 EMA states, window of {K} steps + finalize + allocate (K={len(w.configs)} configurations)",
                   "blocks": len(w.blocks), "coordinates": D, "grad_dtype": w.grad_dtype, "window_steps": K,
                   "gradient_ring": R, "workspace_bytes": nbytes, "launch_shape": {k: (getattr(a, k) or "default") for k in ("chunk_groups", "chunk_slices", "groups_per_wave",
                                                                                        "waves_per_workgroup", "resident_workgroups")}},
        "breakdown_ms": {"begin": round(r["begin"] * 1e3, 3), "first_step": round(step_ms[0], 4), "step_avg": round(avg_ms, 4),
                         "step_min": round(min(steady), 4), "finalize": round(finalize_ms, 3),
                         "allocate": round(r["allocate"] * 1e3, 3)},
        "step_only_elements_per_s": D / (avg_ms * 1e-3),
        "allocation": {"objective": r["obj"], "state_bytes": int(r["mem_used"]), "budget_bytes": int(b_mem)},
        "roofline": {"bound": "hbm", "kernel": "k_step (steady state, launches 2..K)", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": bpe * D, "avg_launch_ms": avg_ms, "launches": len(steady)},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, ring, a.seed, params)
    if not a.no_secondary and a.workload == "llama7b":
        # after the headline window: the pure-stream ceiling of this byte mix, and the steady-state step of the
        # two fp32 layouts the bandwidth target also names (1.3B-shaped decoder, UNet-shaped)
        del theta
        torch.cuda.empty_cache()
        try:                                               # the headline line is printed whatever happens to the extras
            out["roofline"]["practical_ceiling"] = practical_ceiling(w, ring[0], dev)
        except Exception as e:                             # noqa: BLE001
            out["roofline"]["practical_ceiling"] = {"error": repr(e)}
        del ring
        torch.cuda.empty_cache()
        try:
            out["secondary"] = secondary_steps(["gpt_1p3b", "unet"], a, dev)
        except Exception as e:                             # noqa: BLE001
            out["secondary"] = {"error": repr(e)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
