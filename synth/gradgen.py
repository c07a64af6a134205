"""Counter-based synthetic gradient streams (host twin of gradgen.hip).

g_{b,t}[j] = kappa_{b,j} * ( delta_b * n_{b,j} / sqrt(d_b) + sigma_b * xi_{b,t}[j] )

kappa = exp(s_b * zeta), zeta and n fixed standard normals per coordinate, xi fresh
unit-variance noise per step (Gaussian, or Student-t(3)/sqrt(3) for heavy tails).
Every normal is a Box-Muller transform of the bits of a 64-bit mixing function
of (seed, block, stream, step, j), so any element can be produced on its own
and the device generator reproduces the same stream.  Input recipe only: none of
the profiler's arithmetic lives here.
"""
import numpy as np

from .workloads import GAUSS, STUDENT_T3, Workload

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def mix64(x):
    """64-bit finaliser (xor-shift-multiply), vectorised, wrapping arithmetic."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        return x ^ (x >> np.uint64(31))


def stream_key(seed, block, stream, step):
    with np.errstate(over="ignore"):
        k = mix64(np.uint64(seed)) + np.uint64(block)
        k = mix64(k) + ((np.uint64(stream) << np.uint64(32)) | np.uint64(step))
        return mix64(k)


def normal_pair(key, j):
    """Two independent standard normals for each coordinate index in j (uint64 array)."""
    with np.errstate(over="ignore"):
        h = mix64(key + (j + np.uint64(1)) * _GOLD)
    u1 = ((h >> np.uint64(40)).astype(np.float64) + 0.5) * 2.0 ** -24
    u2 = (((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) + 0.5) * 2.0 ** -24
    r = np.sqrt(-2.0 * np.log(u1))
    return r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def block_gradient(seed, block_index, spec, step, lo=0, hi=None):
    """float32 gradient of coordinates [lo, hi) of one block at one step."""
    hi = spec.numel if hi is None else hi
    j = np.arange(lo, hi, dtype=np.uint64)
    zeta, n = normal_pair(stream_key(seed, block_index, 0, 0), j)
    z0, z1 = normal_pair(stream_key(seed, block_index, 1, step), j)
    if spec.noise == STUDENT_T3:
        z2, z3 = normal_pair(stream_key(seed, block_index, 2, step), j)
        xi = z0 / np.sqrt(z1 * z1 + z2 * z2 + z3 * z3)
    else:
        xi = z0
    kappa = np.exp(spec.s * zeta)
    g = kappa * (spec.delta * n / np.sqrt(float(spec.numel)) + spec.sigma * xi)
    return g.astype(np.float32)


def flat_gradient(w: Workload, seed, step, only=None):
    """Whole flat buffer of a workload at one step: float32, or uint16 bf16 bits."""
    out = np.zeros(w.buffer_numel, dtype=np.float32)
    for i, b in enumerate(w.blocks):
        if only is not None and i not in only:
            continue
        out[b.offset:b.offset + b.numel] = block_gradient(seed, i, b, step)
    return f32_to_bf16_bits(out) if w.grad_dtype == "bf16" else out
