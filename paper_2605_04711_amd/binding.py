"""ctypes binding of libbaoc.so: argument marshalling only.

Every step of the path runs inside the library (HIP kernels and its host
code); PyTorch appears here only as the owner of device memory and streams.
The library is loaded from the package directory and built with hipcc when it
is not there; there is no fallback if it cannot be loaded.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_INVALID, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP, ERR_INFEASIBLE, ERR_LIMIT, ERR_STATE = 0, -1, -2, -3, -4, -5, -6, -7
GRAD_F32, GRAD_BF16 = 0, 1
STATIC_WORKSPACE_BYTES = 128 << 20      # BAOC_STATIC_WORKSPACE_BYTES


class Block(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("numel", C.c_uint64), ("rows", C.c_uint32), ("cols", C.c_uint32)]


class ProfileParams(C.Structure):
    _fields_ = [("beta_m", C.c_float), ("beta_v", C.c_float), ("beta_rho", C.c_double), ("eps", C.c_double),
                ("eps_update", C.c_float), ("quant_block", C.c_uint32), ("grad_dtype", C.c_uint32),
                ("chunk_groups", C.c_uint32), ("chunk_slices", C.c_uint32), ("groups_per_wave", C.c_uint32),
                ("waves_per_workgroup", C.c_uint32), ("resident_workgroups", C.c_uint32)]


class Config(C.Structure):
    _fields_ = [("y_a", C.c_uint8), ("y_m", C.c_uint8), ("y_d", C.c_uint8), ("y_f", C.c_uint8), ("bits", C.c_uint8)]


class RiskParams(C.Structure):
    _fields_ = [("gamma", C.c_double), ("A_low", C.c_double), ("A_high", C.c_double),
                ("rho_low", C.c_double), ("rho_high", C.c_double), ("eta_low", C.c_double), ("eta_high", C.c_double),
                ("use_snr_gate", C.c_int32), ("lambda_pref", C.c_double),
                ("pref_mask", C.c_void_p), ("C_raw", C.c_void_p), ("F_raw", C.c_void_p),
                ("compute_F", C.c_int32), ("d_theta_flat", C.c_void_p), ("theta_numel", C.c_uint64),
                ("theta_dtype", C.c_uint32)]


class BlockStats(C.Structure):
    _fields_ = [("numel", C.c_uint64), ("steps", C.c_uint32), ("n_cos", C.c_uint32)] + [
        (n, C.c_double) for n in (
            "rho_bar", "cos_last", "snr", "A", "q10", "q90", "Q16", "Q8", "lQ32", "lQ16", "lQ8",
            "err_m16", "err_v16", "err_m8", "err_v8", "s_A", "s_rho", "s_snr", "s_M", "C_tilde", "s_F",
            "m_sq", "v_l1", "g_sq_last", "C", "F")]

    def asdict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


STAT_FIELDS = [n for n, _ in BlockStats._fields_]


class BaocError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library():
    """dlopen the in-tree libbaoc.so, building it first only when no built library is there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_lib()
    L = C.CDLL(_build.LIB)
    vp, u32, u64, i64, f64 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int64, C.c_double
    L.baoc_profile_params_default.argtypes = [C.POINTER(ProfileParams)]
    L.baoc_profile_params_default.restype = None
    L.baoc_risk_params_default.argtypes = [C.POINTER(RiskParams)]
    L.baoc_risk_params_default.restype = None
    L.baoc_profile_workspace_bytes.argtypes = [C.POINTER(Block), u32, C.POINTER(ProfileParams), C.POINTER(u64)]
    L.baoc_profile_begin.argtypes = [C.POINTER(Block), u32, C.POINTER(ProfileParams), vp, u64, C.POINTER(vp)]
    L.baoc_profile_begin_static.argtypes = [C.POINTER(Block), u32, C.POINTER(ProfileParams), C.POINTER(vp)]
    L.baoc_profile_step.argtypes = [vp, vp, u64, vp]
    L.baoc_profile_finalize.argtypes = [vp, C.POINTER(Config), u32, C.POINTER(RiskParams),
                                        C.POINTER(BlockStats), vp, vp]
    L.baoc_profile_state.argtypes = [vp, u32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    L.baoc_profile_end.argtypes = [vp]
    L.baoc_sample_layout.argtypes = [C.POINTER(Block), u32, f64, C.POINTER(Block), C.POINTER(u64), C.POINTER(u64)]
    L.baoc_sample_begin.argtypes = [C.POINTER(Block), u32, f64, u64, vp, u64, C.POINTER(vp)]
    L.baoc_sample_gather.argtypes = [vp, vp, u64, u32, vp, u64, vp]
    L.baoc_sample_indices.argtypes = [vp, u32, C.POINTER(vp), C.POINTER(u64)]
    L.baoc_sample_end.argtypes = [vp]
    L.baoc_allocate.argtypes = [vp, vp, vp, u32, u32, i64, f64, vp, vp, C.POINTER(f64), C.POINTER(i64), C.POINTER(f64)]
    L.baoc_partition.argtypes = [vp, vp, u32, u32, vp, f64, vp, C.POINTER(u32), C.POINTER(f64)]
    L.baoc_allocate_set_node_limit.argtypes = [u64]
    L.baoc_allocate_set_node_limit.restype = None
    L.baoc_allocate_set_exact_work.argtypes = [u64, u32]
    L.baoc_allocate_set_exact_work.restype = None
    L.baoc_status_string.argtypes = [C.c_int]
    L.baoc_status_string.restype = C.c_char_p
    _lib = L
    return L


def status_string(status):
    return load_library().baoc_status_string(int(status)).decode()


def _check(rc, where):
    if rc != OK:
        raise BaocError(rc, where)


def default_profile_params(**kw):
    p = ProfileParams()
    load_library().baoc_profile_params_default(C.byref(p))
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def default_risk_params(**kw):
    p = RiskParams()
    load_library().baoc_risk_params_default(C.byref(p))
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _block_array(blocks):
    arr = (Block * len(blocks))()
    for i, b in enumerate(blocks):
        if isinstance(b, (tuple, list)):
            o, n = int(b[0]), int(b[1])
            r, c = (int(b[2]), int(b[3])) if len(b) >= 4 else (0, 0)
        else:
            o, n, r, c = int(b.offset), int(b.numel), int(getattr(b, "rows", 0)), int(getattr(b, "cols", 0))
        arr[i] = Block(o, n, r, c)
    return arr


def workspace_bytes(blocks, params=None):
    params = params or default_profile_params()
    out = C.c_uint64()
    arr = _block_array(blocks)
    _check(load_library().baoc_profile_workspace_bytes(arr, len(blocks), C.byref(params), C.byref(out)),
           "baoc_profile_workspace_bytes")
    return out.value


def config_array(configs):
    arr = (Config * len(configs))()
    for i, c in enumerate(configs):
        arr[i] = Config(*[int(x) for x in c])
    return arr


class Profiler:
    """baoc_profile_begin / step / finalize / end around a torch-owned workspace.

    blocks: sequence of (offset, numel[, rows, cols]) or objects with those attributes.
    workspace: optional caller-owned uint8 device tensor of at least workspace_bytes(blocks, params)
    bytes, 256-byte aligned; its previous contents do not matter.  workspace="static" uses the
    library's own per-GPU array instead (baoc_profile_begin_static: no device allocation at all,
    layouts up to STATIC_WORKSPACE_BYTES, one such profiler alive per GPU).
    """

    def __init__(self, blocks, params=None, device="cuda:0", workspace=None, **kw):
        import torch
        self._torch = torch
        self.lib = load_library()
        self.params = params or default_profile_params(**kw)
        self.n_blocks = len(blocks)
        self._blocks = _block_array(blocks)
        nbytes = C.c_uint64()
        _check(self.lib.baoc_profile_workspace_bytes(self._blocks, self.n_blocks, C.byref(self.params), C.byref(nbytes)),
               "baoc_profile_workspace_bytes")
        self.device = torch.device(device)
        self._h = C.c_void_p()
        if isinstance(workspace, str):
            if workspace != "static":
                raise ValueError('workspace must be a tensor, None or "static"')
            self.workspace = None
            with torch.cuda.device(self.device):
                _check(self.lib.baoc_profile_begin_static(self._blocks, self.n_blocks, C.byref(self.params), C.byref(self._h)),
                       "baoc_profile_begin_static")
            return
        if workspace is None:
            workspace = torch.empty(nbytes.value, dtype=torch.uint8, device=self.device)
        elif workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.device != self.device:
            raise TypeError(f"workspace must be a contiguous uint8 tensor on {self.device}")
        self.workspace = workspace
        with torch.cuda.device(self.device):
            _check(self.lib.baoc_profile_begin(self._blocks, self.n_blocks, C.byref(self.params),
                                               self.workspace.data_ptr(), self.workspace.numel(), C.byref(self._h)),
                   "baoc_profile_begin")

    def step(self, grad, stream=None):
        """grad: flat torch tensor on the device, float32 or bfloat16 as given at begin."""
        torch = self._torch
        want = torch.float32 if self.params.grad_dtype == GRAD_F32 else torch.bfloat16
        if grad.dtype != want or not grad.is_contiguous() or grad.device != self.device:
            raise TypeError(f"gradient must be a contiguous {want} tensor on {self.device}")
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        _check(self.lib.baoc_profile_step(self._h, grad.data_ptr(), grad.numel(), s.cuda_stream), "baoc_profile_step")

    def step_raw(self, d_ptr, numel, stream_handle):
        return self.lib.baoc_profile_step(self._h, d_ptr, numel, stream_handle)

    def finalize(self, configs=None, risk_params=None, pref_mask=None, C_raw=None, F_raw=None, theta=None,
                 compute_F=None, stream=None):
        """-> (stats: ctypes array of BlockStats, risk: float64 [N, K] or None).

        theta: flat device tensor of the parameters (float32 or bfloat16, laid out like the gradient
        buffer); when given the distortion C is computed from it.  F is computed for matrix blocks
        unless F_raw is given or compute_F is False."""
        torch = self._torch
        rp = risk_params or default_risk_params()
        keep = []
        if compute_F is not None:
            rp.compute_F = int(bool(compute_F))
        if theta is not None:
            if theta.dtype not in (torch.float32, torch.bfloat16) or not theta.is_contiguous() or theta.device != self.device:
                raise TypeError(f"theta must be a contiguous float32 or bfloat16 tensor on {self.device}")
            keep.append(theta)
            rp.d_theta_flat = theta.data_ptr(); rp.theta_numel = theta.numel()
            rp.theta_dtype = GRAD_F32 if theta.dtype == torch.float32 else GRAD_BF16
        if pref_mask is not None:
            a = np.ascontiguousarray(pref_mask, dtype=np.uint8); keep.append(a); rp.pref_mask = a.ctypes.data
        if C_raw is not None:
            a = np.ascontiguousarray(C_raw, dtype=np.float64); keep.append(a); rp.C_raw = a.ctypes.data
        if F_raw is not None:
            a = np.ascontiguousarray(F_raw, dtype=np.float64); keep.append(a); rp.F_raw = a.ctypes.data
        stats = (BlockStats * self.n_blocks)()
        K = 0 if configs is None else len(configs)
        risk = np.zeros((self.n_blocks, K), np.float64) if K else None
        cfg = config_array(configs) if K else None
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        _check(self.lib.baoc_profile_finalize(self._h, cfg, K, C.byref(rp), stats,
                                              risk.ctypes.data if K else None, s.cuda_stream),
               "baoc_profile_finalize")
        return stats, risk

    def state(self, block):
        """(m, v, g_prev) of one block as torch views into the workspace."""
        torch = self._torch
        pm, pv, pg = C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(self.lib.baoc_profile_state(self._h, block, C.byref(pm), C.byref(pv), C.byref(pg)), "baoc_profile_state")
        if self.workspace is None:
            raise RuntimeError("state views need a torch-owned workspace")
        base = self.workspace.data_ptr()
        n = self._blocks[block].numel
        gsz = 4 if self.params.grad_dtype == GRAD_F32 else 2
        gdt = torch.float32 if gsz == 4 else torch.bfloat16

        def view(ptr, dt, size):
            off = ptr.value - base
            return self.workspace[off:off + n * size].view(dt)
        return view(pm, torch.float32, 4), view(pv, torch.float32, 4), view(pg, gdt, gsz)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self.lib.baoc_profile_end(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Sampler:
    """baoc_sample_* : fixed index sets Omega_i (Sec. 3.1) and the gather into a compact buffer.

    compact_blocks is the layout to hand to Profiler for the compact buffer."""

    def __init__(self, blocks, ratio, seed=0, device="cuda:0"):
        import torch
        self._torch = torch
        self.lib = load_library()
        self.n_blocks = len(blocks)
        self._blocks = _block_array(blocks)
        compact = (Block * self.n_blocks)()
        cn, wb = C.c_uint64(), C.c_uint64()
        _check(self.lib.baoc_sample_layout(self._blocks, self.n_blocks, float(ratio), compact, C.byref(cn), C.byref(wb)),
               "baoc_sample_layout")
        self.compact_blocks = [(b.offset, b.numel, b.rows, b.cols) for b in compact]
        self.compact_numel = cn.value
        self.device = torch.device(device)
        self.workspace = torch.empty(max(wb.value, 256), dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.baoc_sample_begin(self._blocks, self.n_blocks, float(ratio), int(seed),
                                              self.workspace.data_ptr(), self.workspace.numel(), C.byref(self._h)),
                   "baoc_sample_begin")

    def gather(self, grad, out=None, stream=None):
        torch = self._torch
        if grad.dtype not in (torch.float32, torch.bfloat16) or not grad.is_contiguous() or grad.device != self.device:
            raise TypeError(f"gradient must be a contiguous float32 or bfloat16 tensor on {self.device}")
        if out is None:
            out = torch.zeros(self.compact_numel, dtype=grad.dtype, device=self.device)
        if out.dtype != grad.dtype or not out.is_contiguous() or out.device != self.device:
            raise TypeError("compact buffer must match the gradient's dtype and device")
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        _check(self.lib.baoc_sample_gather(self._h, grad.data_ptr(), grad.numel(),
                                           GRAD_F32 if grad.dtype == torch.float32 else GRAD_BF16,
                                           out.data_ptr(), out.numel(), s.cuda_stream), "baoc_sample_gather")
        return out

    def indices(self, block):
        """Omega of one block as an int64 torch view (absolute positions in the flat buffer)."""
        torch = self._torch
        p, n = C.c_void_p(), C.c_uint64()
        _check(self.lib.baoc_sample_indices(self._h, block, C.byref(p), C.byref(n)), "baoc_sample_indices")
        off = p.value - self.workspace.data_ptr()
        return self.workspace[off:off + 8 * n.value].view(torch.int64)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self.lib.baoc_sample_end(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def partition(unit_numel, z, weights=None, alpha=0.01):
    """baoc_partition -> (block id per unit uint32[m], number of blocks, tau)."""
    numel = np.ascontiguousarray(unit_numel, dtype=np.uint64)
    z = np.ascontiguousarray(z, dtype=np.float64)
    m, K = z.shape
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
    ids = np.zeros(m, np.uint32)
    nb, tau = C.c_uint32(), C.c_double()
    rc = load_library().baoc_partition(numel.ctypes.data, z.ctypes.data, m, K, None if w is None else w.ctypes.data,
                                       float(alpha), ids.ctypes.data, C.byref(nb), C.byref(tau))
    _check(rc, "baoc_partition")
    return ids, nb.value, tau.value


def allocate(risk, mem_cost_bytes, time_cost, mem_budget_bytes, time_budget_sum, forbidden=None):
    """baoc_allocate -> (choice uint32[N], objective, mem, time). Raises BaocError on failure."""
    risk = np.ascontiguousarray(risk, dtype=np.float64)
    N, K = risk.shape
    mem = np.ascontiguousarray(mem_cost_bytes, dtype=np.int64).reshape(N, K)
    tc = np.ascontiguousarray(time_cost, dtype=np.float64).reshape(N, K)
    fb = None if forbidden is None else np.ascontiguousarray(forbidden, dtype=np.uint8).reshape(N, K)
    choice = np.zeros(N, np.uint32)
    obj, om, ot = C.c_double(), C.c_int64(), C.c_double()
    rc = load_library().baoc_allocate(risk.ctypes.data, mem.ctypes.data, tc.ctypes.data, N, K, int(mem_budget_bytes),
                                      float(time_budget_sum), None if fb is None else fb.ctypes.data,
                                      choice.ctypes.data, C.byref(obj), C.byref(om), C.byref(ot))
    _check(rc, "baoc_allocate")
    return choice, obj.value, om.value, ot.value
