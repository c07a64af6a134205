"""ctypes front end of the CPU oracle (baoc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing here touches the HIP library and the
HIP library never touches this.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "baoc_oracle.c")
_LIB = os.path.join(_HERE, "libbaoc_oracle.so")

# -ffp-contract=off: every fp32 operation of the state update is rounded once, as written
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force=False):
    """Compile the oracle with gcc (seconds). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.run(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"], check=True)
    return _LIB


class Stats(C.Structure):
    _fields_ = [("numel", C.c_uint64), ("steps", C.c_uint32), ("n_cos", C.c_uint32)] + [
        (n, C.c_double) for n in (
            "rho_bar", "cos_last", "snr", "A", "q10", "q90",
            "Q16", "Q8", "lQ32", "lQ16", "lQ8",
            "err_m16", "err_v16", "err_m8", "err_v8",
            "s_A", "s_rho", "s_snr", "s_M", "C_tilde", "s_F",
            "m_sq", "v_l1", "g_sq_last", "C", "F")]

    def asdict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


STAT_FIELDS = [n for n, _ in Stats._fields_]


class RiskParams(C.Structure):
    _fields_ = [(n, C.c_double) for n in (
        "gamma", "A_low", "A_high", "rho_low", "rho_high", "eta_low", "eta_high")] + [
        ("use_snr_gate", C.c_int), ("lambda_pref", C.c_double)]


def default_risk_params(**kw):
    """gamma of Eq. 1 and the anchors of App. A."""
    import math
    p = RiskParams(0.1, math.log(2.0), math.log(10.0), 0.2, 0.6, 0.0, 2.0, 1, 0.0)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, u64, u32, f32, f64, i64 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_float, C.c_double, C.c_int64
        L.orc_block_new.restype = vp
        L.orc_block_new.argtypes = [u64, f32, f32, f64, f64, f32, u32]
        L.orc_block_free.argtypes = [vp]
        for n in ("orc_block_m", "orc_block_v", "orc_block_p"):
            getattr(L, n).restype = C.POINTER(C.c_float)
            getattr(L, n).argtypes = [vp]
        L.orc_block_step_f32.argtypes = [vp, vp]
        L.orc_block_step_bf16.argtypes = [vp, vp]
        L.orc_block_finalize.argtypes = [vp, C.POINTER(RiskParams), f64, f64, C.POINTER(Stats)]
        L.orc_block_structure_residual.restype = f64
        L.orc_block_structure_residual.argtypes = [vp, u32, u32]
        L.orc_block_distortion.restype = f64
        L.orc_block_distortion.argtypes = [vp, vp]
        L.orc_sample_count.restype = u64
        L.orc_sample_count.argtypes = [u64, f64]
        L.orc_sample_indices.restype = None
        L.orc_sample_indices.argtypes = [u64, u64, u64, u32, vp]
        L.orc_sample_matrix_shape.argtypes = [u32, u32, f64, C.POINTER(u32), C.POINTER(u32)]
        L.orc_sample_indices_matrix.restype = None
        L.orc_sample_indices_matrix.argtypes = [u32, u32, u32, u32, u64, u32, vp]
        L.orc_bf16_round.restype = f32
        L.orc_bf16_round.argtypes = [f32]
        L.orc_q8_code.restype = f32
        L.orc_q8_code.argtypes = [f32, f32, f32]
        L.orc_quantile.restype = f64
        L.orc_quantile.argtypes = [vp, u64, f64]
        L.orc_agg.restype = f64
        L.orc_agg.argtypes = [C.c_int] * 5
        L.orc_phi.restype = f64
        L.orc_phi.argtypes = [C.POINTER(Stats), C.c_char_p, C.c_int, C.POINTER(RiskParams)]
        for n in ("orc_allocate_brute", "orc_allocate_dp", "orc_allocate_bnb"):
            getattr(L, n).argtypes = [vp, vp, vp, u32, u32, i64, f64, vp, vp,
                                      C.POINTER(f64), C.POINTER(i64), C.POINTER(f64)]
        L.orc_allocate_bnb_set_node_limit.restype = None
        L.orc_allocate_bnb_set_node_limit.argtypes = [u64]
        L.orc_allocate_bnb_last_nodes.restype = u64
        L.orc_allocate_bnb_last_nodes.argtypes = []
        L.orc_integerise.argtypes = [vp, vp, vp, u32, u32, i64, f64, vp, vp, vp, vp, C.POINTER(i64)]
        _lib = L
    return _lib


ORC_OK, ORC_INVALID, ORC_INFEASIBLE, ORC_TOO_BIG = 0, -1, -5, -6


class Block:
    """Profiler state of one parameter block; step() takes that block's slice."""

    def __init__(self, numel, beta_m=0.9, beta_v=0.999, beta_rho=0.9, eps=1e-12, eps_u=1e-8, qb=256):
        self.numel = int(numel)
        self._h = lib().orc_block_new(self.numel, beta_m, beta_v, beta_rho, eps, eps_u, qb)
        if not self._h:
            raise MemoryError("oracle block")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_block_free(self._h)
            self._h = None

    def step(self, g):
        """g: float32 array, or uint16 array holding bf16 bit patterns."""
        g = np.ascontiguousarray(g)
        assert g.size == self.numel
        if g.dtype == np.float32:
            rc = lib().orc_block_step_f32(self._h, g.ctypes.data)
        elif g.dtype == np.uint16:
            rc = lib().orc_block_step_bf16(self._h, g.ctypes.data)
        else:
            raise TypeError("gradient dtype must be float32 or uint16 (bf16 bits)")
        if rc:
            raise MemoryError("oracle step")

    def _arr(self, fn):
        p = fn(self._h)
        return np.ctypeslib.as_array(p, shape=(self.numel,)).copy()

    @property
    def m(self):
        return self._arr(lib().orc_block_m)

    @property
    def v(self):
        return self._arr(lib().orc_block_v)

    @property
    def p(self):
        return self._arr(lib().orc_block_p)

    def structure_residual(self, rows, cols):
        """Eq. 7 on v-hat viewed as rows x cols; 0 for non-matrix blocks."""
        return lib().orc_block_structure_residual(self._h, int(rows), int(cols))

    def distortion(self, theta):
        """Eq. 6 with the block's parameters theta (float32, or uint16 bf16 bits)."""
        theta = np.ascontiguousarray(theta)
        if theta.dtype == np.uint16:
            theta = (theta.astype(np.uint32) << np.uint32(16)).view(np.float32)
        theta = np.ascontiguousarray(theta, dtype=np.float32)
        assert theta.size == self.numel
        return lib().orc_block_distortion(self._h, theta.ctypes.data)

    def finalize(self, rp=None, C_raw=0.0, F_raw=0.0):
        rp = rp or default_risk_params()
        st = Stats()
        if lib().orc_block_finalize(self._h, C.byref(rp), C_raw, F_raw, C.byref(st)):
            raise MemoryError("oracle finalize")
        return st


class Profiler:
    """All blocks of a layout over one flat gradient buffer.

    blocks: sequence of (offset, numel) in elements of the flat buffer.
    """

    def __init__(self, blocks, **params):
        self.blocks = [(int(o), int(n)) for o, n in blocks]
        self.state = [Block(n, **params) for _, n in self.blocks]

    def step(self, flat, only=None):
        idx = range(len(self.blocks)) if only is None else only
        for i in idx:
            o, n = self.blocks[i]
            self.state[i].step(flat[o:o + n])

    def finalize(self, configs, rp=None, pref_mask=None, C_raw=None, F_raw=None, only=None):
        """-> (list of Stats, risk table Phi[N,K] as float64)."""
        rp = rp or default_risk_params()
        idx = list(range(len(self.blocks)) if only is None else only)
        stats, rows = [], []
        for i in idx:
            st = self.state[i].finalize(rp, 0.0 if C_raw is None else float(C_raw[i]),
                                        0.0 if F_raw is None else float(F_raw[i]))
            stats.append(st)
            rows.append([phi(st, c, bool(pref_mask[k]) if pref_mask is not None else False, rp)
                         for k, c in enumerate(configs)])
        return stats, np.array(rows, dtype=np.float64).reshape(len(idx), len(configs))


def sample_count(d, s):
    """|Omega| = ceil(s d), clamped to [1, d] (Sec. 3.1)."""
    return lib().orc_sample_count(int(d), float(s))


def sample_indices(d, s, seed, block):
    """The fixed index set Omega of one block (ascending uint64 array)."""
    k = sample_count(d, s)
    out = np.zeros(k, np.uint64)
    lib().orc_sample_indices(int(d), k, int(seed), int(block), out.ctypes.data)
    return out


def sample_matrix_shape(rows, cols, s):
    """(r, c) of the sampled sub-matrix of a rows x cols block, or None when the sample has no matrix form."""
    r, c = C.c_uint32(), C.c_uint32()
    if not lib().orc_sample_matrix_shape(int(rows), int(cols), float(s), C.byref(r), C.byref(c)):
        return None
    return r.value, c.value


def sample_indices_block(numel, rows, cols, s, seed, block):
    """Omega of one block as positions inside the block, and the compact block's (rows, cols): the product
    form for matrix blocks (sub-matrix, row-major), the flat stratified draw otherwise ((0, 0))."""
    shape = sample_matrix_shape(rows, cols, s) if rows and cols else None
    if shape is None:
        return sample_indices(numel, s, seed, block), (0, 0)
    r, c = shape
    out = np.zeros(r * c, np.uint64)
    lib().orc_sample_indices_matrix(int(rows), int(cols), r, c, int(seed), int(block), out.ctypes.data)
    return out, (r, c)


def phi(stats, cfg, preferred=False, rp=None):
    rp = rp or default_risk_params()
    return lib().orc_phi(C.byref(stats), bytes(bytearray(int(x) for x in cfg)), int(preferred), C.byref(rp))


def agg(cfg):
    return lib().orc_agg(*[int(x) for x in cfg])


def bf16_round(x):
    return lib().orc_bf16_round(float(x))


def q8_code(x, a, L):
    return lib().orc_q8_code(float(x), float(a), float(L))


def quantile(x, q):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return lib().orc_quantile(x.ctypes.data, x.size, q)


def _allocate(fn, risk, mem, time, mem_budget, time_budget_sum, forbidden):
    risk = np.ascontiguousarray(risk, dtype=np.float64)
    N, K = risk.shape
    mem = np.ascontiguousarray(mem, dtype=np.int64).reshape(N, K)
    time = np.ascontiguousarray(time, dtype=np.float64).reshape(N, K)
    fb = None if forbidden is None else np.ascontiguousarray(forbidden, dtype=np.uint8).reshape(N, K)
    choice = np.zeros(N, dtype=np.uint32)
    obj, om, ot = C.c_double(), C.c_int64(), C.c_double()
    rc = fn(risk.ctypes.data, mem.ctypes.data, time.ctypes.data, N, K, int(mem_budget),
            float(time_budget_sum), None if fb is None else fb.ctypes.data, choice.ctypes.data,
            C.byref(obj), C.byref(om), C.byref(ot))
    return rc, choice, obj.value, om.value, ot.value


def allocate_brute(risk, mem, time, mem_budget, time_budget_sum, forbidden=None):
    """Exhaustive K^N enumeration -> (rc, choice, objective, mem, time)."""
    return _allocate(lib().orc_allocate_brute, risk, mem, time, mem_budget, time_budget_sum, forbidden)


def allocate_dp(risk, mem, time, mem_budget, time_budget_sum, forbidden=None):
    """Textbook two-row knapsack dynamic programme (small integer resources)."""
    return _allocate(lib().orc_allocate_dp, risk, mem, time, mem_budget, time_budget_sum, forbidden)


def allocate_bnb(risk, mem, time, mem_budget, time_budget_sum, forbidden=None, node_limit=0):
    """Depth-first branch and bound in lexicographic order, for instances the other two cannot
    reach.  node_limit: search nodes after which the call gives up with ORC_TOO_BIG (0 = default)."""
    lib().orc_allocate_bnb_set_node_limit(int(node_limit))
    return _allocate(lib().orc_allocate_bnb, risk, mem, time, mem_budget, time_budget_sum, forbidden)


def allocate_bnb_nodes():
    """Search nodes of the last allocate_bnb call."""
    return lib().orc_allocate_bnb_last_nodes()


def integerise(risk, mem, time, mem_budget, time_budget_sum, forbidden=None):
    risk = np.ascontiguousarray(risk, dtype=np.float64)
    N, K = risk.shape
    mem = np.ascontiguousarray(mem, dtype=np.int64).reshape(N, K)
    time = np.ascontiguousarray(time, dtype=np.float64).reshape(N, K)
    fb = None if forbidden is None else np.ascontiguousarray(forbidden, dtype=np.uint8).reshape(N, K)
    phi_i = np.zeros((N, K), np.int64)
    tau = np.zeros((N, K), np.int64)
    ok = np.zeros((N, K), np.uint8)
    bt = C.c_int64()
    rc = lib().orc_integerise(risk.ctypes.data, mem.ctypes.data, time.ctypes.data, N, K, int(mem_budget),
                              float(time_budget_sum), None if fb is None else fb.ctypes.data,
                              phi_i.ctypes.data, tau.ctypes.data, ok.ctypes.data, C.byref(bt))
    return rc, phi_i, tau, ok, bt.value
