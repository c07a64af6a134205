"""Launches the device gradient generator (csrc/gradgen.hip) on torch-owned buffers."""
import ctypes as C
import os
import subprocess

from .workloads import Workload

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "gradgen.hip")
LIB = os.path.join(_HERE, "libbaoc_gradgen.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

PROBE_SRC = os.path.join(_HERE, "csrc", "memprobe.hip")
PROBE_LIB = os.path.join(_HERE, "libbaoc_memprobe.so")

_lib = None
_probe = None


def build_probe():
    subprocess.run(["hipcc", *FLAGS, "-o", PROBE_LIB, PROBE_SRC], check=True, stderr=subprocess.DEVNULL)
    return PROBE_LIB


def probe_lib():
    """The pure-stream probe (csrc/memprobe.hip): the step kernel's traffic mix with no arithmetic."""
    global _probe
    if _probe is None:
        if not os.path.exists(PROBE_LIB):
            build_probe()
        _probe = C.CDLL(PROBE_LIB)
        _probe.synth_mix_stream.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    return _probe


def build_lib():
    subprocess.run(["hipcc", *FLAGS, "-o", LIB, SRC], check=True, stderr=subprocess.DEVNULL)
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build_lib()
        _lib = C.CDLL(LIB)
        _lib.synth_fill_block.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32,
                                          C.c_float, C.c_float, C.c_float, C.c_uint32, C.c_void_p]
    return _lib


def new_buffer(w: Workload, device="cuda:0"):
    import torch
    dt = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    return torch.zeros(w.buffer_numel, dtype=dt, device=device)


def fill(w: Workload, buf, seed, step, only=None):
    """Write step `step` of the workload's stream into the flat device tensor `buf` (current stream)."""
    import torch
    L = lib()
    esz = buf.element_size()
    dtype = 1 if w.grad_dtype == "bf16" else 0
    st = torch.cuda.current_stream(buf.device).cuda_stream
    base = buf.data_ptr()
    for i, b in enumerate(w.blocks):
        if only is not None and i not in only:
            continue
        rc = L.synth_fill_block(base + b.offset * esz, dtype, b.numel, int(seed), i, int(step),
                                b.delta, b.sigma, b.s, b.noise, st)
        if rc:
            raise RuntimeError(f"synth_fill_block: hip error {rc}")
    return buf
