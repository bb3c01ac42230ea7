"""ctypes binding of libgpd.so: same names as the C ABI in include/gpd.h.

Argument marshalling only: every function here hands device pointers of torch tensors
(torch is used for device memory and streams) to the library and returns what the library
wrote.  There is no fallback: without the built library or without a GPU the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpd.so")

GPD_MAX_P = 64
GPD_OK, GPD_E_INVALID, GPD_E_SHAPE, GPD_E_POINTS, GPD_E_TOO_FEW, GPD_E_DECODE_FAIL, \
    GPD_E_WORKSPACE, GPD_E_DEVICE, GPD_E_UNSUPPORTED, GPD_E_VERIFY = range(10)
GPD_F32, GPD_BF16, GPD_F32_SPLIT = 0, 1, 2
GPD_SUB_AUTO, GPD_SUB_U_VN, GPD_SUB_V_UM = 0, 1, 2
GPD_DEC_FIRST_K, GPD_DEC_LSQ_ALL = 0, 1
GPD_STEP_FORWARD, GPD_STEP_BACKWARD_UPDATE = 0, 1
GPD_STEP_FUSE_SIGMOID = 0x100
GPD_CORRECT_NONE, GPD_CORRECT_ELEMENTS, GPD_CORRECT_NODES, GPD_CORRECT_ELEMENTS_L1 = 0, 1, 2, 3
GPD_STACK_WEIGHTS, GPD_STACK_FORWARD, GPD_STACK_BACKWARD = 0, 1, 2
GPD_LAYOUT_PACKED, GPD_LAYOUT_SPREAD = 0, 1

STATUS_NAMES = ["OK", "E_INVALID", "E_SHAPE", "E_POINTS", "E_TOO_FEW", "E_DECODE_FAIL",
                "E_WORKSPACE", "E_DEVICE", "E_UNSUPPORTED", "E_VERIFY"]

EXPORTS = [
    "gpd_plan", "gpd_plan_info", "gpd_plan_strides", "gpd_plan_tables", "gpd_plan_destroy", "gpd_encode",
    "gpd_worker_products", "gpd_decode", "gpd_layer_create", "gpd_layer_info",
    "gpd_layer_encode_weights", "gpd_layer_decode_weights", "gpd_coded_layer_step",
    "gpd_layer_workspace_view", "gpd_layer_destroy", "gpd_sigmoid_fwd", "gpd_sigmoid_bwd", "gpd_l2_delta",
    "gpd_host_code", "gpd_host_decode_matrices", "gpd_last_error", "gpd_version",
    "gpd_locate_nodes", "gpd_layer_locate_nodes", "gpd_layer_regenerate", "gpd_layer_project",
    "gpd_host_parity_check", "gpd_host_locate_nodes", "gpd_verify_decode",
    "gpd_row_mean", "gpd_sigmoid_bwd_sparse", "gpd_decode_static",
    "gpd_timing_tag", "gpd_timing_collect", "gpd_timing_reset", "gpd_mlp_step",
]


class GpdError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"gpd status {STATUS_NAMES[status] if 0 <= status < 10 else status}: {msg}")
        self.status = status


class _Problem(C.Structure):
    _fields_ = [("N1", C.c_int64), ("N0", C.c_int64), ("Nc", C.c_int64),
                ("m", C.c_int32), ("n", C.c_int32), ("d", C.c_int32), ("P", C.c_int32),
                ("points", C.POINTER(C.c_double)),
                ("worker_dtype", C.c_int32), ("subst", C.c_int32),
                ("rho_detect", C.c_double), ("abs_floor", C.c_double),
                ("hip_stream", C.c_void_p), ("stack_layout", C.c_int32)]


class _Located(C.Structure):
    _fields_ = [("node", C.c_int32), ("row", C.c_int32), ("col", C.c_int32),
                ("magnitude", C.c_float)]


class _Report(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_present", C.c_int32),
                ("n_screened", C.c_int64), ("n_flagged", C.c_int64),
                ("n_located", C.c_int64), ("n_failed", C.c_int64),
                ("node_err_count", C.c_int32 * GPD_MAX_P),
                ("max_syndrome_ratio", C.c_float), ("reserved", C.c_int32),
                ("located_cap", C.c_int64), ("located", C.POINTER(_Located))]


class _NodeReport(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_present", C.c_int32), ("n_bad", C.c_int32),
                ("exhaustive", C.c_int32), ("bad", C.c_uint8 * GPD_MAX_P), ("wild", C.c_uint8 * GPD_MAX_P),
                ("energy", C.c_double), ("syndrome_energy", C.c_double), ("residual", C.c_double),
                ("threshold", C.c_double)]


class _VerifyReport(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_checked", C.c_int32), ("n_value_mismatch", C.c_int32),
                ("locations_agree", C.c_int32), ("bad", C.c_uint8 * GPD_MAX_P), ("max_ratio", C.c_double)]


class _LayerDesc(C.Structure):
    _fields_ = [("N_out", C.c_int64), ("N_in", C.c_int64), ("batch", C.c_int64),
                ("m", C.c_int32), ("n", C.c_int32), ("d1", C.c_int32), ("d2", C.c_int32),
                ("P", C.c_int32),
                ("points", C.POINTER(C.c_double)),
                ("worker_dtype", C.c_int32), ("subst", C.c_int32),
                ("rho_detect", C.c_double), ("abs_floor", C.c_double),
                ("hip_stream", C.c_void_p)]


_lib = None


def load_library():
    """Loads libgpd.so (built in-tree by paper_1811_10751_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_1811_10751_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.gpd_plan.argtypes = [C.POINTER(_Problem), C.POINTER(vp)]
    lib.gpd_plan_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(sz)]
    lib.gpd_plan_strides.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.gpd_plan_tables.argtypes = [vp, vp, vp, vp, vp]
    lib.gpd_plan_destroy.argtypes = [vp]
    lib.gpd_plan_destroy.restype = None
    lib.gpd_encode.argtypes = [vp, vp, i64, vp, i64, vp, vp]
    lib.gpd_worker_products.argtypes = [vp, vp, vp, vp]
    lib.gpd_decode.argtypes = [vp, vp, vp, i32, i32, vp, i64, vp, sz, C.POINTER(_Report)]
    lib.gpd_decode_static.argtypes = [vp, vp, vp, i32, i32, vp, i64, C.POINTER(_Report)]
    lib.gpd_layer_create.argtypes = [C.POINTER(_LayerDesc), C.POINTER(vp)]
    lib.gpd_layer_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64),
                                   C.POINTER(i64), C.POINTER(sz)]
    lib.gpd_layer_encode_weights.argtypes = [vp, vp, i64, vp]
    lib.gpd_layer_decode_weights.argtypes = [vp, vp, vp, vp, i64]
    lib.gpd_coded_layer_step.argtypes = [vp, i32, vp, vp, vp, C.c_float, C.c_float, vp, vp, i32,
                                         vp, sz, C.POINTER(_Report)]
    lib.gpd_layer_workspace_view.argtypes = [vp, i32, C.POINTER(sz), C.POINTER(i64), C.POINTER(i64)]
    lib.gpd_layer_destroy.argtypes = [vp]
    lib.gpd_layer_destroy.restype = None
    lib.gpd_sigmoid_fwd.argtypes = [vp, vp, i64, vp]
    lib.gpd_sigmoid_bwd.argtypes = [vp, vp, vp, i64, vp]
    lib.gpd_l2_delta.argtypes = [vp, vp, C.c_float, vp, i64, vp]
    lib.gpd_row_mean.argtypes = [vp, i64, i64, vp, vp]
    lib.gpd_sigmoid_bwd_sparse.argtypes = [vp, vp, vp, C.c_float, C.c_float, vp, i64, i64, vp]
    lib.gpd_host_code.argtypes = [i32, i32, i32, i32, i32, vp, C.POINTER(i32), vp, vp, vp, vp]
    lib.gpd_host_decode_matrices.argtypes = [i32, i32, i32, i32, i32, vp, vp, i32, vp, vp,
                                             C.POINTER(i32)]
    lib.gpd_locate_nodes.argtypes = [vp, vp, vp, vp, sz, C.POINTER(_NodeReport), vp]
    lib.gpd_layer_locate_nodes.argtypes = [vp, i32, vp, vp, vp, sz, C.POINTER(_NodeReport), vp]
    lib.gpd_layer_regenerate.argtypes = [vp, vp, vp, i32]
    lib.gpd_layer_project.argtypes = [vp, vp, vp]
    lib.gpd_host_parity_check.argtypes = [i32, i32, vp, vp, vp, C.POINTER(i32)]
    lib.gpd_host_locate_nodes.argtypes = [i32, i32, vp, vp, vp, C.c_double, i64, C.c_double, C.c_double,
                                          vp, C.POINTER(_NodeReport)]
    lib.gpd_verify_decode.argtypes = [vp, vp, vp, i32, vp, vp, i64, i32, vp, sz, C.POINTER(_VerifyReport)]
    lib.gpd_mlp_step.argtypes = [C.POINTER(vp), i32, C.POINTER(vp), vp, vp, C.c_float, C.c_float,
                                 C.POINTER(vp), C.POINTER(vp), C.POINTER(sz)]
    lib.gpd_timing_tag.argtypes = [i32]
    lib.gpd_timing_collect.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.gpd_timing_reset.argtypes = []
    lib.gpd_last_error.restype = C.c_char_p
    lib.gpd_version.restype = C.c_char_p
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int:
            fn.restype = C.c_int32
    _lib = lib
    return lib


def _check(st: int, ok=(GPD_OK,)):
    if st not in ok:
        raise GpdError(st, load_library().gpd_last_error().decode())
    return st


def _ptr(t):
    """Device (or host) pointer of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream_handle(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _require_f32_cuda(t, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32):
        raise TypeError(f"{name} must be a float32 CUDA tensor")


@dataclass
class Report:
    status: int = 0
    n_present: int = 0
    n_screened: int = 0
    n_flagged: int = 0
    n_located: int = 0
    n_failed: int = 0
    node_err_count: np.ndarray | None = None
    max_syndrome_ratio: float = 0.0
    located: list = field(default_factory=list)   # (node, row, col, magnitude), sorted


def _make_report(cap: int):
    buf = (_Located * max(cap, 1))()
    rep = _Report()
    rep.located = C.cast(buf, C.POINTER(_Located))
    rep.located_cap = cap
    return rep, buf


def _read_report(rep: _Report, buf, P: int, listed: bool = True) -> Report:
    # with node-level correction whole nodes are located and no per-element list is written
    n = int(min(rep.n_located, rep.located_cap)) if listed else 0
    return Report(status=rep.status, n_present=rep.n_present, n_screened=rep.n_screened,
                  n_flagged=rep.n_flagged, n_located=rep.n_located, n_failed=rep.n_failed,
                  node_err_count=np.array(rep.node_err_count[:P], dtype=np.int64),
                  max_syndrome_ratio=float(rep.max_syndrome_ratio),
                  located=[(buf[i].node, buf[i].row, buf[i].col, buf[i].magnitude) for i in range(n)])


def _present_array(present, P):
    if present is None:
        return None
    arr = np.ascontiguousarray(np.asarray(present, dtype=np.uint8))
    if arr.shape != (P,):
        raise ValueError("present must have P entries")
    return arr


class Plan:
    """Owns a gpd_plan_t*."""

    def __init__(self, handle, problem: _Problem, keep):
        self.handle = handle
        self.problem = problem
        self._keep = keep
        lib = load_library()
        K, t, ws = C.c_int32(), C.c_int32(), C.c_size_t()
        _check(lib.gpd_plan_info(handle, C.byref(K), C.byref(t), C.byref(ws)))
        self.K, self.t_max, self.workspace_bytes = K.value, t.value, ws.value
        self.m, self.n, self.d, self.P = problem.m, problem.n, problem.d, problem.P
        self.N1, self.N0, self.Nc = problem.N1, problem.N0, problem.Nc
        self.worker_dtype = problem.worker_dtype
        sa, sb, sc = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib.gpd_plan_strides(handle, C.byref(sa), C.byref(sb), C.byref(sc)))
        self.strides = {"A": sa.value, "B": sb.value, "C": sc.value}
        self.layout = problem.stack_layout

    def stack_shape(self, which):
        return {"A": (self.P, self.N1 // self.m, self.N0 // self.n),
                "B": (self.P, self.N0 // self.n, self.Nc // self.d),
                "C": (self.P, self.N1 // self.m, self.Nc // self.d)}[which]

    def alloc_stack(self, which, device, dtype=None):
        """Uninitialised coded stack At ("A"), Bt ("B") or Ct ("C") in the plan's layout: a
        [P, rows, cols] view whose node blocks lie the plan's stride apart."""
        import torch
        if dtype is None:
            dtype = torch.float32 if which == "C" or self.worker_dtype != GPD_BF16 else torch.bfloat16
        P, rows, cols = self.stack_shape(which)
        stride = self.strides[which]
        base = torch.empty(max(P * stride, 1), dtype=dtype, device=device)
        return base.as_strided((P, rows, cols), (stride, cols, 1))

    def clone_stack(self, t, which="C"):
        """A copy of the coded stack t in the plan's layout (torch's clone would pack it)."""
        out = self.alloc_stack(which, t.device, t.dtype)
        out.copy_(t)
        return out

    def stack_ok(self, t, which):
        """True if tensor t is a coded stack of this plan: shape and node stride match."""
        P, rows, cols = self.stack_shape(which)
        if tuple(t.shape) != (P, rows, cols):
            return False
        if rows * cols == 0:
            return True
        want = (self.strides[which], cols, 1)
        return all(t.shape[i] == 1 or t.stride(i) == want[i] for i in range(3))

    def tables(self):
        lib = load_library()
        pts = np.zeros(self.P)
        eA = np.zeros(self.m * self.n, dtype=np.int32)
        eB = np.zeros(self.n * self.d, dtype=np.int32)
        eC = np.zeros(self.m * self.d, dtype=np.int32)
        _check(lib.gpd_plan_tables(self.handle, pts.ctypes.data, eA.ctypes.data, eB.ctypes.data,
                                   eC.ctypes.data))
        return pts, eA.reshape(self.m, self.n), eB.reshape(self.n, self.d), eC.reshape(self.m, self.d)

    def close(self):
        if self.handle:
            load_library().gpd_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gpd_plan(N1, N0, Nc, m, n, d, P, points=None, worker_dtype=GPD_F32, subst=GPD_SUB_AUTO,
             rho_detect=0.0, abs_floor=0.0, stream=None, layout=GPD_LAYOUT_PACKED) -> Plan:
    lib = load_library()
    pr = _Problem()
    pr.N1, pr.N0, pr.Nc, pr.m, pr.n, pr.d, pr.P = N1, N0, Nc, m, n, d, P
    keep = None
    if points is not None:
        keep = np.ascontiguousarray(np.asarray(points, dtype=np.float64))
        if keep.shape != (P,):
            raise ValueError("points must have P entries")
        pr.points = keep.ctypes.data_as(C.POINTER(C.c_double))
    pr.worker_dtype, pr.subst = worker_dtype, subst
    pr.rho_detect, pr.abs_floor = rho_detect, abs_floor
    pr.hip_stream = _stream_handle(stream)
    pr.stack_layout = layout
    h = C.c_void_p()
    _check(lib.gpd_plan(C.byref(pr), C.byref(h)))
    return Plan(h, pr, keep)


def gpd_encode(plan: Plan, A=None, B=None, At=None, Bt=None):
    """At[P, N1/m, N0/n], Bt[P, N0/n, Nc/d] (allocated here if not given)."""
    import torch
    lib = load_library()
    dt = torch.bfloat16 if plan.worker_dtype == GPD_BF16 else torch.float32
    lda = ldb = 0
    if A is not None:
        _require_f32_cuda(A, "A")
        if A.dim() != 2 or A.shape != (plan.N1, plan.N0) or A.stride(1) != 1:
            raise ValueError("A must be N1 x N0 with unit column stride")
        lda = A.stride(0)
        if At is None:
            At = plan.alloc_stack("A", A.device, dt)
    if B is not None:
        _require_f32_cuda(B, "B")
        if B.dim() != 2 or B.shape != (plan.N0, plan.Nc) or B.stride(1) != 1:
            raise ValueError("B must be N0 x Nc with unit column stride")
        ldb = B.stride(0)
        if Bt is None:
            Bt = plan.alloc_stack("B", B.device, dt)
    for t, which in ((At, "A"), (Bt, "B")):
        if t is not None and (not plan.stack_ok(t, which) or t.dtype != dt):
            raise ValueError("coded stacks must have the plan's layout and the worker dtype")
    _check(lib.gpd_encode(plan.handle, _ptr(A), lda, _ptr(B), ldb,
                          _ptr(At) if A is not None else None, _ptr(Bt) if B is not None else None))
    return At, Bt


def gpd_worker_products(plan: Plan, At, Bt, Ct=None):
    import torch
    lib = load_library()
    dt = torch.bfloat16 if plan.worker_dtype == GPD_BF16 else torch.float32
    if At.dtype != dt or Bt.dtype != dt or not plan.stack_ok(At, "A") or not plan.stack_ok(Bt, "B"):
        raise ValueError("At/Bt do not match the plan")
    if Ct is None:
        Ct = plan.alloc_stack("C", At.device)
    elif Ct.dtype != torch.float32 or not plan.stack_ok(Ct, "C"):
        raise ValueError("Ct does not match the plan")
    _check(lib.gpd_worker_products(plan.handle, _ptr(At), _ptr(Bt), _ptr(Ct)))
    return Ct


def gpd_decode(plan: Plan, Ct, present=None, mode=GPD_DEC_FIRST_K, correct_errors=False, C_out=None,
               workspace=None, want_report=True, located_cap=4096, raise_on_fail=False):
    """Returns (C, Report or None)."""
    import torch
    lib = load_library()
    _require_f32_cuda(Ct, "Ct")
    if not plan.stack_ok(Ct, "C"):
        raise ValueError("Ct does not match the plan (shape or node stride)")
    if C_out is None:
        C_out = torch.empty((plan.N1, plan.Nc), dtype=torch.float32, device=Ct.device)
    elif tuple(C_out.shape) != (plan.N1, plan.Nc) or C_out.stride(1) != 1 or C_out.dtype != torch.float32:
        raise ValueError("C_out does not match the plan")
    pres = _present_array(present, plan.P)
    ws_ptr, ws_bytes = None, 0
    if correct_errors:
        if workspace is None:
            workspace = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=Ct.device)
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    rep = buf = None
    if want_report:
        rep, buf = _make_report(located_cap)
    st = lib.gpd_decode(plan.handle, _ptr(Ct), _ptr(pres), mode, int(correct_errors),
                        _ptr(C_out), C_out.stride(0), ws_ptr, ws_bytes,
                        C.byref(rep) if rep is not None else None)
    _check(st, ok=(GPD_OK,) if raise_on_fail else (GPD_OK, GPD_E_DECODE_FAIL))
    return C_out, (_read_report(rep, buf, plan.P, int(correct_errors) != GPD_CORRECT_NODES)
                   if rep is not None else None)


def gpd_decode_static(plan: Plan, Ct, C_out, present=None, mode=GPD_DEC_FIRST_K, correct_errors=False,
                      want_report=True, located_cap=4096, raise_on_fail=False):
    """gpd_decode without a workspace: the library's fixed scratch array is used.  C_out must be
    given (this call allocates nothing on the device).  Returns (C_out, Report or None)."""
    import torch
    lib = load_library()
    _require_f32_cuda(Ct, "Ct")
    if not plan.stack_ok(Ct, "C"):
        raise ValueError("Ct does not match the plan (shape or node stride)")
    if tuple(C_out.shape) != (plan.N1, plan.Nc) or C_out.stride(1) != 1 or C_out.dtype != torch.float32:
        raise ValueError("C_out does not match the plan")
    pres = _present_array(present, plan.P)
    rep = buf = None
    if want_report:
        rep, buf = _make_report(located_cap)
    st = lib.gpd_decode_static(plan.handle, _ptr(Ct), _ptr(pres), mode, int(correct_errors),
                               _ptr(C_out), C_out.stride(0), C.byref(rep) if rep is not None else None)
    _check(st, ok=(GPD_OK,) if raise_on_fail else (GPD_OK, GPD_E_DECODE_FAIL))
    return C_out, (_read_report(rep, buf, plan.P) if rep is not None else None)


# ------------------------------------------------------------------ coded DNN layer


class Layer:
    """Owns a gpd_layer_t*."""

    def __init__(self, handle, desc: _LayerDesc, keep):
        self.handle, self.desc, self._keep = handle, desc, keep
        lib = load_library()
        kf, kb, r, c, ws = C.c_int32(), C.c_int32(), C.c_int64(), C.c_int64(), C.c_size_t()
        _check(lib.gpd_layer_info(handle, C.byref(kf), C.byref(kb), C.byref(r), C.byref(c), C.byref(ws)))
        self.Kf, self.Kb, self.wt_rows, self.wt_cols, self.workspace_bytes = \
            kf.value, kb.value, r.value, c.value, ws.value
        self.N_out, self.N_in, self.batch, self.P = desc.N_out, desc.N_in, desc.batch, desc.P
        self.worker_dtype = desc.worker_dtype
        self._ws = None

    def workspace(self, device):
        import torch
        if self._ws is None:
            self._ws = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8, device=device)
        return self._ws

    def view(self, which, device):
        """fp32 tensor [P, rows, cols] aliasing one of the per-node intermediates in the workspace
        (0 X~, 1 S~, 2 Delta~, 3 C~, 4 Dhat, 5 Xhat); 6: int32 [2], the exponents E of Dhat and
        Xhat when those are held as fp16 planes (hi + lo) * 2^E."""
        import torch
        lib = load_library()
        off, r, c = C.c_size_t(), C.c_int64(), C.c_int64()
        ws = self.workspace(device)
        fp16 = lib.gpd_layer_workspace_view(self.handle, 6, C.byref(off), C.byref(r), C.byref(c)) == GPD_OK
        if which == 6:
            if not fp16:
                raise ValueError("this layer holds no fp16 planes")
            return ws[off.value:off.value + 8].view(torch.int32)
        _check(lib.gpd_layer_workspace_view(self.handle, which, C.byref(off), C.byref(r), C.byref(c)))
        n = self.P * r.value * c.value
        if which >= 4 and fp16:
            # two fp16 planes (hi, lo) of the operand / 2^E, each [P][cols/16][rows][16]
            return ws[off.value:off.value + 4 * n].view(torch.float16).view(2, self.P, c.value // 16, r.value, 16)
        if which in (0, 2) and self.worker_dtype == GPD_BF16:
            return ws[off.value:off.value + 2 * n].view(torch.bfloat16).view(self.P, r.value, c.value)
        if which >= 4 and self.worker_dtype != GPD_F32 and self.batch % 64 == 0:
            # three bf16 planes (hi, mid, lo), each [P][cols/16][rows][16]
            return ws[off.value:off.value + 6 * n].view(torch.bfloat16).view(3, self.P, c.value // 16, r.value, 16)
        return ws[off.value:off.value + 4 * n].view(torch.float32).view(self.P, r.value, c.value)

    def workspace_delta(self, device):
        """The error Delta of this layer (N_out x batch) where gpd_mlp_step leaves it."""
        import torch
        off, r, c = C.c_size_t(), C.c_int64(), C.c_int64()
        _check(load_library().gpd_layer_workspace_view(self.handle, 7, C.byref(off), C.byref(r), C.byref(c)))
        ws = self.workspace(device)
        return ws[off.value:off.value + 4 * r.value * c.value].view(torch.float32).view(r.value, c.value)[:self.N_out]

    def close(self):
        if self.handle:
            load_library().gpd_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gpd_layer_create(N_out, N_in, batch, m, n, d1, d2, P, points=None, worker_dtype=GPD_F32,
                     subst=GPD_SUB_AUTO, rho_detect=0.0, abs_floor=0.0, stream=None) -> Layer:
    lib = load_library()
    d = _LayerDesc()
    d.N_out, d.N_in, d.batch, d.m, d.n, d.d1, d.d2, d.P = N_out, N_in, batch, m, n, d1, d2, P
    keep = None
    if points is not None:
        keep = np.ascontiguousarray(np.asarray(points, dtype=np.float64))
        d.points = keep.ctypes.data_as(C.POINTER(C.c_double))
    d.worker_dtype, d.subst, d.rho_detect, d.abs_floor = worker_dtype, subst, rho_detect, abs_floor
    d.hip_stream = _stream_handle(stream)
    h = C.c_void_p()
    _check(lib.gpd_layer_create(C.byref(d), C.byref(h)))
    return Layer(h, d, keep)


def gpd_layer_encode_weights(layer: Layer, W, Wt=None):
    import torch
    _require_f32_cuda(W, "W")
    if tuple(W.shape) != (layer.N_out, layer.N_in) or W.stride(1) != 1:
        raise ValueError("W must be N_out x N_in")
    if Wt is None:
        Wt = torch.empty((layer.P, layer.wt_rows, layer.wt_cols), dtype=torch.float32, device=W.device)
    _check(load_library().gpd_layer_encode_weights(layer.handle, _ptr(W), W.stride(0), _ptr(Wt)))
    return Wt


def gpd_layer_decode_weights(layer: Layer, Wt, present=None, W=None):
    import torch
    _require_f32_cuda(Wt, "Wt")
    if W is None:
        W = torch.empty((layer.N_out, layer.N_in), dtype=torch.float32, device=Wt.device)
    pres = _present_array(present, layer.P)
    _check(load_library().gpd_layer_decode_weights(layer.handle, _ptr(Wt), _ptr(pres), _ptr(W), W.stride(0)))
    return W


def gpd_coded_layer_step(layer: Layer, phase, Wt, X, Dlt=None, eta=0.0, decay=0.0, out=None,
                         present=None, correct_errors=False, want_report=False, located_cap=4096,
                         skip_output=False, fuse_sigmoid=False):
    """FORWARD: returns (S, report); BACKWARD_UPDATE: returns (C or None, report); Wt updated in place.
    fuse_sigmoid: the element-wise step after the decode is applied in the same pass (FORWARD:
    the logistic function of S is returned; BACKWARD_UPDATE: C o X o (1 - X))."""
    import torch
    lib = load_library()
    _require_f32_cuda(Wt, "Wt")
    _require_f32_cuda(X, "X")
    if tuple(Wt.shape) != (layer.P, layer.wt_rows, layer.wt_cols) or not Wt.is_contiguous():
        raise ValueError("Wt does not match the layer")
    if tuple(X.shape) != (layer.N_in, layer.batch) or not X.is_contiguous():
        raise ValueError("X must be contiguous N_in x batch")
    if phase == GPD_STEP_BACKWARD_UPDATE:
        _require_f32_cuda(Dlt, "Dlt")
        if tuple(Dlt.shape) != (layer.N_out, layer.batch) or not Dlt.is_contiguous():
            raise ValueError("Dlt must be contiguous N_out x batch")
    rows = layer.N_out if phase == GPD_STEP_FORWARD else layer.N_in
    if out is None and not skip_output:
        out = torch.empty((rows, layer.batch), dtype=torch.float32, device=X.device)
    if out is not None and (tuple(out.shape) != (rows, layer.batch) or not out.is_contiguous()):
        raise ValueError("out has the wrong shape")
    ws = layer.workspace(X.device)
    pres = _present_array(present, layer.P)
    rep = buf = None
    if want_report:
        rep, buf = _make_report(located_cap)
    st = lib.gpd_coded_layer_step(layer.handle, phase | (GPD_STEP_FUSE_SIGMOID if fuse_sigmoid else 0),
                                  _ptr(Wt), _ptr(X), _ptr(Dlt), eta, decay,
                                  _ptr(out), _ptr(pres), int(correct_errors),
                                  ws.data_ptr(), ws.numel(), C.byref(rep) if rep is not None else None)
    _check(st, ok=(GPD_OK, GPD_E_DECODE_FAIL))
    return out, (_read_report(rep, buf, layer.P, int(correct_errors) != GPD_CORRECT_NODES)
                 if rep is not None else None)


def gpd_mlp_step(layers, Wts, X, Y, eta, decay, acts):
    """One whole training iteration of the network `layers` on the small-batch path (see gpd.h).
    acts: list of float32 CUDA tensors N_out(l) x batch, written.  Returns False, launching
    nothing, if the network is outside what the fused path covers."""
    lib = load_library()
    n = len(layers)
    _require_f32_cuda(X, "X")
    _require_f32_cuda(Y, "Y")
    if tuple(X.shape) != (layers[0].N_in, layers[0].batch) or not X.is_contiguous():
        raise ValueError("X must be contiguous N_in x batch")
    if tuple(Y.shape) != (layers[-1].N_out, layers[-1].batch) or not Y.is_contiguous():
        raise ValueError("Y must be contiguous N_out x batch")
    for L, Wt, a in zip(layers, Wts, acts):
        _require_f32_cuda(Wt, "Wt")
        _require_f32_cuda(a, "acts")
        if tuple(Wt.shape) != (L.P, L.wt_rows, L.wt_cols) or not Wt.is_contiguous():
            raise ValueError("Wt does not match the layer")
        if tuple(a.shape) != (L.N_out, L.batch) or not a.is_contiguous():
            raise ValueError("acts[l] must be contiguous N_out x batch")
    wss = [L.workspace(X.device) for L in layers]
    arr = lambda vals: (C.c_void_p * n)(*vals)
    st = lib.gpd_mlp_step(arr([L.handle.value for L in layers]), n, arr([w.data_ptr() for w in Wts]),
                          _ptr(X), _ptr(Y), eta, decay, arr([a.data_ptr() for a in acts]),
                          arr([w.data_ptr() for w in wss]), (C.c_size_t * n)(*[w.numel() for w in wss]))
    if st in (GPD_E_UNSUPPORTED, GPD_E_SHAPE):
        return False
    _check(st)
    return True


# ------------------------------------------------------------------ node-level faults


@dataclass
class NodeReport:
    status: int = 0
    n_present: int = 0
    bad: tuple = ()                 # node indices found erroneous, ascending
    wild: tuple = ()                # nodes that held a non-finite or huge value
    exhaustive: bool = True
    energy: float = 0.0
    syndrome_energy: float = 0.0
    residual: float = 0.0
    threshold: float = 0.0


def _read_node_report(rep: _NodeReport, P: int) -> NodeReport:
    return NodeReport(rep.status, rep.n_present, tuple(p for p in range(P) if rep.bad[p]),
                      tuple(p for p in range(P) if rep.wild[p]), bool(rep.exhaustive), rep.energy,
                      rep.syndrome_energy, rep.residual, rep.threshold)


def _gram_buffer(want, P, K, pres):
    if not want:
        return None
    ns = P if pres is None else int(np.count_nonzero(pres))
    return np.zeros((max(ns - K, 0), max(ns - K, 0)))


def gpd_locate_nodes(plan: Plan, Ct, present=None, workspace=None, want_gram=False):
    """NodeReport, or (NodeReport, gram) with want_gram."""
    import torch
    lib = load_library()
    _require_f32_cuda(Ct, "Ct")
    if not plan.stack_ok(Ct, "C"):
        raise ValueError("Ct does not match the plan (shape or node stride)")
    if workspace is None:
        workspace = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=Ct.device)
    pres = _present_array(present, plan.P)
    rep = _NodeReport()
    gram = _gram_buffer(want_gram, plan.P, plan.K, pres)
    st = lib.gpd_locate_nodes(plan.handle, _ptr(Ct), _ptr(pres), workspace.data_ptr(), workspace.numel(),
                              C.byref(rep), gram.ctypes.data if gram is not None and gram.size else None)
    _check(st, ok=(GPD_OK, GPD_E_DECODE_FAIL))
    out = _read_node_report(rep, plan.P)
    return (out, gram) if want_gram else out


@dataclass
class VerifyReport:
    status: int = 0
    n_checked: int = 0
    n_value_mismatch: int = 0
    locations_agree: bool = True
    bad: tuple = ()
    max_ratio: float = 0.0


def gpd_verify_decode(plan: Plan, Ct, C_dec, present=None, mode=GPD_DEC_FIRST_K, bad=(), n_check=0,
                      workspace=None) -> VerifyReport:
    """Second, independent decode of n_check (default P) pre-decided values of C_dec; status
    GPD_E_VERIFY in the report on disagreement."""
    import torch
    lib = load_library()
    _require_f32_cuda(Ct, "Ct")
    _require_f32_cuda(C_dec, "C")
    if not plan.stack_ok(Ct, "C"):
        raise ValueError("Ct does not match the plan (shape or node stride)")
    if tuple(C_dec.shape) != (plan.N1, plan.Nc) or C_dec.stride(1) != 1:
        raise ValueError("C does not match the plan")
    if workspace is None:
        workspace = torch.empty(max(plan.workspace_bytes, 1 << 20), dtype=torch.uint8, device=Ct.device)
    pres = _present_array(present, plan.P)
    mask = None
    if bad is not None and len(tuple(bad)):
        mask = np.zeros(plan.P, dtype=np.uint8)
        for p in bad:
            mask[int(p)] = 1
    rep = _VerifyReport()
    st = lib.gpd_verify_decode(plan.handle, _ptr(Ct), _ptr(pres), mode, _ptr(mask), _ptr(C_dec), C_dec.stride(0),
                               n_check, workspace.data_ptr(), workspace.numel(), C.byref(rep))
    _check(st, ok=(GPD_OK, GPD_E_VERIFY))
    return VerifyReport(rep.status, rep.n_checked, rep.n_value_mismatch, bool(rep.locations_agree),
                        tuple(p for p in range(plan.P) if rep.bad[p]), rep.max_ratio)


def gpd_layer_locate_nodes(layer: Layer, which, stack, present=None, want_gram=False):
    lib = load_library()
    _require_f32_cuda(stack, "stack")
    shapes = {GPD_STACK_WEIGHTS: (layer.wt_rows, layer.wt_cols),
              GPD_STACK_FORWARD: (layer.wt_rows, layer.batch // layer.desc.d1),
              GPD_STACK_BACKWARD: (layer.wt_cols, layer.batch // layer.desc.d2)}
    if which not in shapes or tuple(stack.shape) != (layer.P,) + shapes[which] or not stack.is_contiguous():
        raise ValueError("stack does not match the layer")
    ws = layer.workspace(stack.device)
    pres = _present_array(present, layer.P)
    rep = _NodeReport()
    K = {GPD_STACK_WEIGHTS: layer.desc.m * layer.desc.n, GPD_STACK_FORWARD: layer.Kf,
         GPD_STACK_BACKWARD: layer.Kb}[which]
    gram = _gram_buffer(want_gram, layer.P, K, pres)
    st = lib.gpd_layer_locate_nodes(layer.handle, which, _ptr(stack), _ptr(pres), ws.data_ptr(), ws.numel(),
                                    C.byref(rep), gram.ctypes.data if gram is not None and gram.size else None)
    _check(st, ok=(GPD_OK, GPD_E_DECODE_FAIL))
    out = _read_node_report(rep, layer.P)
    return (out, gram) if want_gram else out


def _weights_ok(layer: Layer, Wt):
    _require_f32_cuda(Wt, "Wt")
    if tuple(Wt.shape) != (layer.P, layer.wt_rows, layer.wt_cols) or not Wt.is_contiguous():
        raise ValueError("Wt does not match the layer")


def gpd_layer_regenerate(layer: Layer, Wt, bad, mode=GPD_DEC_LSQ_ALL):
    """bad: iterable of node indices; their blocks of Wt are recomputed in place."""
    lib = load_library()
    _weights_ok(layer, Wt)
    mask = np.zeros(layer.P, dtype=np.uint8)
    for p in bad:
        mask[int(p)] = 1
    _check(lib.gpd_layer_regenerate(layer.handle, _ptr(Wt), mask.ctypes.data, mode))
    return Wt


def gpd_layer_project(layer: Layer, Wt, present=None):
    lib = load_library()
    _weights_ok(layer, Wt)
    pres = _present_array(present, layer.P)
    _check(lib.gpd_layer_project(layer.handle, _ptr(Wt), _ptr(pres)))
    return Wt


def gpd_host_parity_check(P, K, points=None, present=None):
    """H[n_present-K, n_present] as the library computes it; no GPU needed."""
    lib = load_library()
    pres = _present_array(present, P)
    ns = P if pres is None else int(np.count_nonzero(pres))
    if ns < K:
        raise GpdError(GPD_E_TOO_FEW, "too few responses")
    H = np.zeros((ns - K, ns))
    pin = None if points is None else np.ascontiguousarray(np.asarray(points, dtype=np.float64))
    nsv = C.c_int32()
    _check(lib.gpd_host_parity_check(P, K, _ptr(pin), _ptr(pres), H.ctypes.data, C.byref(nsv)))
    return H


def gpd_host_locate_nodes(P, K, gram, energy, n_codewords, rho, abs_floor=0.0, points=None, present=None,
                          forced=None) -> NodeReport:
    """The host half of gpd_locate_nodes on a Gram matrix given in the basis of gpd_host_parity_check."""
    lib = load_library()
    pres = _present_array(present, P)
    pin = None if points is None else np.ascontiguousarray(np.asarray(points, dtype=np.float64))
    g = np.ascontiguousarray(np.asarray(gram, dtype=np.float64))
    f = None
    if forced is not None:
        f = np.zeros(P, dtype=np.uint8)
        f[list(forced)] = 1
    rep = _NodeReport()
    st = lib.gpd_host_locate_nodes(P, K, _ptr(pin), _ptr(pres), g.ctypes.data if g.size else None,
                                   float(energy), int(n_codewords), float(rho), float(abs_floor),
                                   _ptr(f), C.byref(rep))
    _check(st, ok=(GPD_OK, GPD_E_DECODE_FAIL))
    return _read_node_report(rep, P)


def gpd_sigmoid_fwd(s, y=None, stream=None):
    import torch
    y = torch.empty_like(s) if y is None else y
    _check(load_library().gpd_sigmoid_fwd(_ptr(s), _ptr(y), s.numel(), _stream_handle(stream)))
    return y


def gpd_sigmoid_bwd(c, y, out=None, stream=None):
    import torch
    out = torch.empty_like(c) if out is None else out
    _check(load_library().gpd_sigmoid_bwd(_ptr(c), _ptr(y), _ptr(out), c.numel(), _stream_handle(stream)))
    return out


def gpd_l2_delta(y, yhat, scale, out=None, stream=None):
    import torch
    out = torch.empty_like(yhat) if out is None else out
    _check(load_library().gpd_l2_delta(_ptr(y), _ptr(yhat), scale, _ptr(out), yhat.numel(),
                                       _stream_handle(stream)))
    return out


def gpd_row_mean(y, out=None, stream=None):
    import torch
    _require_f32_cuda(y, "y")
    if y.dim() != 2 or not y.is_contiguous():
        raise ValueError("y must be a contiguous matrix")
    if out is None:
        out = torch.empty(y.shape[0], dtype=torch.float32, device=y.device)
    _check(load_library().gpd_row_mean(_ptr(y), y.shape[0], y.shape[1], _ptr(out), _stream_handle(stream)))
    return out


def gpd_sigmoid_bwd_sparse(c, y, rho_hat, rho, scale, out=None, stream=None):
    import torch
    for t, name in ((c, "c"), (y, "y"), (rho_hat, "rho_hat")):
        _require_f32_cuda(t, name)
    if c.shape != y.shape or y.dim() != 2 or rho_hat.numel() != y.shape[0] or not (c.is_contiguous() and y.is_contiguous()):
        raise ValueError("shapes do not match")
    if out is None:
        out = torch.empty_like(c)
    _check(load_library().gpd_sigmoid_bwd_sparse(_ptr(c), _ptr(y), _ptr(rho_hat), rho, scale, _ptr(out), y.shape[0],
                                                 y.shape[1], _stream_handle(stream)))
    return out


def gpd_host_code(m, n, d, P, subst=GPD_SUB_AUTO, points=None):
    """(K, eA[m,n], eB[n,d], eC[m,d], points[P]) from the library's host code; no GPU needed."""
    lib = load_library()
    K = C.c_int32()
    eA = np.zeros(m * n, dtype=np.int32)
    eB = np.zeros(n * d, dtype=np.int32)
    eC = np.zeros(m * d, dtype=np.int32)
    pts = np.zeros(P)
    pin = None if points is None else np.ascontiguousarray(np.asarray(points, dtype=np.float64))
    _check(lib.gpd_host_code(m, n, d, P, subst, _ptr(pin), C.byref(K), eA.ctypes.data, eB.ctypes.data,
                             eC.ctypes.data, pts.ctypes.data))
    return K.value, eA.reshape(m, n), eB.reshape(n, d), eC.reshape(m, d), pts


def gpd_host_decode_matrices(m, n, d, P, subst=GPD_SUB_AUTO, points=None, present=None, first_k=False,
                             want_H=True):
    """(D[m*d, n_present], H[n_present-K, n_present] or None); no GPU needed."""
    lib = load_library()
    K = gpd_host_code(m, n, d, P, subst, points)[0]
    pres = _present_array(present, P)
    ns = P if pres is None else int(np.count_nonzero(pres))
    if ns < K:
        raise GpdError(GPD_E_TOO_FEW, "too few responses")
    D = np.zeros((m * d, ns))
    H = np.zeros((ns - K, ns)) if want_H else None
    pin = None if points is None else np.ascontiguousarray(np.asarray(points, dtype=np.float64))
    nsv = C.c_int32()
    _check(lib.gpd_host_decode_matrices(m, n, d, P, subst, _ptr(pin), _ptr(pres), int(first_k),
                                        D.ctypes.data, _ptr(H), C.byref(nsv)))
    return D, H


def gpd_timing_tag(tag: int):
    """Kernels launched by the library from now on are timed one by one under `tag` (< 0: off)."""
    _check(load_library().gpd_timing_tag(int(tag)))


def gpd_timing_collect(tag: int):
    """(sum of the durations in ms, number of launches) of the kernels recorded under `tag`."""
    ms, n = C.c_double(), C.c_int32()
    _check(load_library().gpd_timing_collect(int(tag), C.byref(ms), C.byref(n)))
    return ms.value, n.value


def gpd_timing_reset():
    _check(load_library().gpd_timing_reset())


def gpd_version() -> str:
    return load_library().gpd_version().decode()
