"""Thin ctypes binding of libsconv.so: same names as include/sconv.h, argument
marshalling only.  PyTorch appears only as the owner of device buffers and
streams.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsconv.so")
_lib = None

SCONV_OK = 0
ERR = {"NULL": -1, "DESC": -2, "CSR": -3, "BATCH": -4, "CAPACITY": -5, "PLAN": -6, "HIP": -7, "NOMEM": -8, "RANGE": -9}


class sconv_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("C", "H", "W", "K", "R", "S", "stride", "pad", "groups")]


class sconv_plan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kernel", "nt", "cb", "waves", "cg", "rows_w", "t", "band", "strip", "splits")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class sconv_machine(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("dense_flops", "hbm_bytes_per_s", "alpha", "beta", "fma_flops",
                                          "lds_bytes_per_s", "lds_bytes_per_fma", "lane_efficiency", "t_fixed")]


class sconv_prediction(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("flops_dense", "bytes_act", "bytes_w", "density", "alpha", "t_dense",
                                          "t_sparse_compute", "t_sparse_bw", "t_sparse", "speedup",
                                          "effective_flops", "actual_flops", "x_upper", "x_lower")] + \
               [("bandwidth_bound", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class sconv_balance(C.Structure):
    _fields_ = [("nnz", C.c_int64), ("stream_entries", C.c_int64)] + \
               [(n, C.c_double) for n in ("wave_mean", "wave_max", "simd_max", "workgroup_mean", "workgroup_max")]


EXPORTS = ["sconv_create_csr", "sconv_create_csr_from_arrays", "sconv_csr_info", "sconv_csr_export",
           "sconv_csr_unpack", "sconv_forward", "sconv_forward_fused", "sconv_last_hip_error", "sconv_destroy_csr", "sconv_strerror",
           "sconv_machine_gfx950", "sconv_model_predict", "sconv_gsl_decide", "sconv_csr_balance",
           "sconv_fc_forward", "sconv_fc_plan", "sconv_tune", "sconv_fc_tune", "sconv_rank_plans",
           "sconv_lower_offsets", "sconv_model_predict_lowered", "sconv_forward_noalloc"]
NOALLOC_SCRATCH_BYTES = 64 << 20
LAYOUT_CHW, LAYOUT_HWC = 0, 1
GSL_ACTIONS = ("exclude", "prune", "stop", "restore_dense")


class SconvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1608_01409_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int64)
        L.sconv_create_csr.argtypes = [C.POINTER(sconv_desc), vp, C.POINTER(sconv_plan), C.POINTER(vp)]
        L.sconv_create_csr_from_arrays.argtypes = [C.POINTER(sconv_desc), vp, vp, vp, C.POINTER(sconv_plan), C.POINTER(vp)]
        L.sconv_csr_info.argtypes = [vp, i64p, C.POINTER(i32), C.POINTER(i32), C.POINTER(sconv_plan)]
        L.sconv_csr_export.argtypes = [vp, vp, vp, vp, i64p]
        L.sconv_csr_unpack.argtypes = [vp, i32, vp, vp, vp, i64p]
        L.sconv_forward.argtypes = [vp, vp, vp, i32, vp]
        L.sconv_forward_noalloc.argtypes = [vp, vp, vp, i32, vp]
        L.sconv_forward_fused.argtypes = [vp, vp, vp, i32, vp, i32, vp]
        L.sconv_fc_forward.argtypes = [vp, vp, vp, i32, vp, i32, vp]
        L.sconv_fc_plan.argtypes = [vp, i32, C.POINTER(sconv_plan)]
        L.sconv_tune.argtypes = [vp, vp, vp, i32, i32, vp]
        L.sconv_rank_plans.argtypes = [vp, i32, i32, C.POINTER(sconv_plan), C.POINTER(i32)]
        L.sconv_fc_tune.argtypes = [vp, vp, vp, i32, i32, vp]
        L.sconv_last_hip_error.argtypes = [vp]
        L.sconv_destroy_csr.argtypes = [vp]
        L.sconv_destroy_csr.restype = None
        L.sconv_strerror.argtypes = [C.c_int]
        L.sconv_strerror.restype = C.c_char_p
        L.sconv_machine_gfx950.argtypes = [C.POINTER(sconv_machine)]
        L.sconv_machine_gfx950.restype = None
        L.sconv_model_predict.argtypes = [C.POINTER(sconv_desc), i32, C.c_double, vp, C.POINTER(sconv_machine),
                                          C.POINTER(sconv_prediction)]
        L.sconv_model_predict_lowered.argtypes = L.sconv_model_predict.argtypes
        L.sconv_lower_offsets.argtypes = [C.POINTER(sconv_desc), i32, vp, vp, vp, C.POINTER(i32), C.POINTER(i32)]
        L.sconv_gsl_decide.argtypes = [C.POINTER(sconv_desc), i32, C.c_double, i32, C.POINTER(sconv_machine),
                                       C.POINTER(i32), C.POINTER(sconv_prediction)]
        L.sconv_csr_balance.argtypes = [C.c_void_p, C.POINTER(sconv_balance)]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().sconv_strerror(status).decode()


def _check(status, where):
    if status != SCONV_OK:
        raise SconvError(status, where)


def make_desc(layer) -> sconv_desc:
    return sconv_desc(*(int(getattr(layer, n)) for n in ("C", "H", "W", "K", "R", "S", "stride", "pad", "groups")))


def make_plan(plan) -> sconv_plan | None:
    if plan is None:
        return None
    if isinstance(plan, sconv_plan):
        return plan
    return sconv_plan(*(int(plan.get(n, 0)) for n, _ in sconv_plan._fields_))


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Csr:
    """Owner of one sconv_csr handle."""

    def __init__(self, handle, layer):
        self._h = C.c_void_p(handle)
        self.layer = layer
        self._destroy = lib().sconv_destroy_csr   # module globals may be gone when __del__ runs at exit

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h


def sconv_create_csr(layer, dense_w: np.ndarray, plan=None) -> Csr:
    w = np.ascontiguousarray(dense_w, dtype=np.float32)
    d = make_desc(layer)
    p = make_plan(plan)
    out = C.c_void_p()
    _check(lib().sconv_create_csr(C.byref(d), _np_ptr(w), C.byref(p) if p is not None else None, C.byref(out)),
           "sconv_create_csr")
    return Csr(out.value, layer)


def sconv_create_csr_from_arrays(layer, rowptr, colidx, values, plan=None) -> Csr:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    values = np.ascontiguousarray(values, dtype=np.float32)
    d = make_desc(layer)
    p = make_plan(plan)
    out = C.c_void_p()
    _check(lib().sconv_create_csr_from_arrays(C.byref(d), _np_ptr(rowptr), _np_ptr(colidx), _np_ptr(values),
                                              C.byref(p) if p is not None else None, C.byref(out)),
           "sconv_create_csr_from_arrays")
    return Csr(out.value, layer)


def sconv_csr_info(csr: Csr):
    nnz, oh, ow, plan = C.c_int64(), C.c_int32(), C.c_int32(), sconv_plan()
    _check(lib().sconv_csr_info(csr.handle, C.byref(nnz), C.byref(oh), C.byref(ow), C.byref(plan)), "sconv_csr_info")
    return {"nnz": nnz.value, "OH": oh.value, "OW": ow.value, "plan": plan.as_dict()}


def _export(fn, csr: Csr, *pre):
    n = C.c_int64(0)
    rc = fn(csr.handle, *pre, None, None, None, C.byref(n))
    if rc not in (SCONV_OK, ERR["CAPACITY"], ERR["NULL"]):
        raise SconvError(rc, "export")
    nnz = n.value
    rowptr = np.zeros(csr.layer.K + 1, dtype=np.int32)
    off = np.zeros(max(nnz, 1), dtype=np.int32)
    val = np.zeros(max(nnz, 1), dtype=np.float32)
    n = C.c_int64(nnz)
    _check(fn(csr.handle, *pre, _np_ptr(rowptr), _np_ptr(off), _np_ptr(val), C.byref(n)), "export")
    return rowptr, off[:nnz], val[:nnz]


def sconv_csr_export(csr: Csr):
    return _export(lib().sconv_csr_export, csr)


def sconv_csr_unpack(csr: Csr, which: int):
    return _export(lib().sconv_csr_unpack, csr, C.c_int32(which))


def _conv_buffers(csr: Csr, x, out, stream):
    """Checks the input tensor, allocates or checks the output, picks the stream: (N, out, stream)."""
    import torch

    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    L = csr.layer
    assert tuple(x.shape[1:]) == (L.C, L.H, L.W), (tuple(x.shape), L)
    N = x.shape[0]
    info = sconv_csr_info(csr)
    if out is None:
        out = torch.empty((N, L.K, info["OH"], info["OW"]), dtype=torch.float32, device=x.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    assert tuple(out.shape) == (N, L.K, info["OH"], info["OW"])
    return N, out, stream if stream is not None else torch.cuda.current_stream(x.device)


def _fc_buffers(csr: Csr, x_t, out_t, bias, stream):
    import torch

    L = csr.layer
    assert x_t.is_cuda and x_t.dtype == torch.float32 and x_t.is_contiguous() and x_t.dim() == 2 and x_t.shape[0] == L.C
    N = x_t.shape[1]
    if out_t is None:
        out_t = torch.empty((L.K, N), dtype=torch.float32, device=x_t.device)
    assert out_t.is_cuda and out_t.dtype == torch.float32 and out_t.is_contiguous() and tuple(out_t.shape) == (L.K, N)
    _check_bias(csr, bias)
    return N, out_t, stream if stream is not None else torch.cuda.current_stream(x_t.device)


def _check_bias(csr: Csr, bias):
    import torch

    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous() and tuple(bias.shape) == (csr.layer.K,)


def sconv_forward(csr: Csr, x, out=None, stream=None):
    """x: contiguous fp32 CUDA tensor [N,C,H,W]; returns/overwrites out [N,K,OH,OW] on the same device."""
    import torch

    N, out, s = _conv_buffers(csr, x, out, stream)
    with torch.cuda.device(x.device):
        rc = lib().sconv_forward(csr.handle, C.c_void_p(x.data_ptr()), C.c_void_p(out.data_ptr()), N,
                                 C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_forward (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out


def sconv_forward_noalloc(csr: Csr, x, out, stream=None):
    """sconv_forward without any allocation: `out` must be given, and the handle prepared by an earlier
    sconv_forward call with the same batch size."""
    import torch

    assert out is not None
    N, out, s = _conv_buffers(csr, x, out, stream)
    with torch.cuda.device(x.device):
        rc = lib().sconv_forward_noalloc(csr.handle, C.c_void_p(x.data_ptr()), C.c_void_p(out.data_ptr()), N,
                                         C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_forward_noalloc (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out


def sconv_rank_plans(csr: Csr, N: int, max_plans: int = 8) -> list:
    """The tilings sconv_tune would time for batch size N, the cost model's choice first."""
    room = 8 if max_plans < 1 else min(int(max_plans), 32)
    plans = (sconv_plan * room)()
    count = C.c_int32(0)
    _check(lib().sconv_rank_plans(csr.handle, N, int(max_plans), plans, C.byref(count)), "sconv_rank_plans")
    return [plans[i].as_dict() for i in range(count.value)]


def sconv_tune(csr: Csr, x, out=None, max_plans=8, stream=None):
    """Times the best-ranked tilings for this batch size on x and keeps the fastest; returns the output."""
    import torch

    N, out, s = _conv_buffers(csr, x, out, stream)
    with torch.cuda.device(x.device):
        rc = lib().sconv_tune(csr.handle, C.c_void_p(x.data_ptr()), C.c_void_p(out.data_ptr()), N, int(max_plans),
                              C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_tune (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out


def sconv_forward_fused(csr: Csr, x, bias=None, relu=False, out=None, stream=None):
    """sconv_forward followed, inside the kernel where it can, by out = max(out + bias[k], 0); bias: fp32 CUDA
    tensor [K] or None."""
    import torch

    N, out, s = _conv_buffers(csr, x, out, stream)
    _check_bias(csr, bias)
    with torch.cuda.device(x.device):
        rc = lib().sconv_forward_fused(csr.handle, C.c_void_p(x.data_ptr()), C.c_void_p(out.data_ptr()), N,
                                       C.c_void_p(bias.data_ptr()) if bias is not None else None, int(bool(relu)),
                                       C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_forward_fused (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out


def fc_layer(C_in: int, K: int):
    """The layer description of a fully connected layer with weights [K][C_in]."""
    from .workloads import Layer
    return Layer(f"fc{C_in}x{K}", C_in, 1, 1, K, 1, 1, 1, 0, 1)


def sconv_fc_plan(csr: Csr, N: int) -> dict:
    p = sconv_plan()
    _check(lib().sconv_fc_plan(csr.handle, N, C.byref(p)), "sconv_fc_plan")
    return p.as_dict()


def sconv_fc_forward(csr: Csr, x_t, bias=None, relu=False, out_t=None, stream=None):
    """x_t: contiguous fp32 CUDA tensor [C][N] (feature-major); returns/overwrites out_t [K][N]."""
    import torch

    N, out_t, s = _fc_buffers(csr, x_t, out_t, bias, stream)
    with torch.cuda.device(x_t.device):
        rc = lib().sconv_fc_forward(csr.handle, C.c_void_p(x_t.data_ptr()), C.c_void_p(out_t.data_ptr()), N,
                                    C.c_void_p(bias.data_ptr()) if bias is not None else None, int(bool(relu)),
                                    C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_fc_forward (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out_t


def sconv_fc_tune(csr: Csr, x_t, out_t=None, max_plans=8, stream=None):
    """Times the best-ranked tilings of the fully connected layer for this batch size; returns the output."""
    import torch

    N, out_t, s = _fc_buffers(csr, x_t, out_t, None, stream)
    with torch.cuda.device(x_t.device):
        rc = lib().sconv_fc_tune(csr.handle, C.c_void_p(x_t.data_ptr()), C.c_void_p(out_t.data_ptr()), N, int(max_plans),
                                 C.c_void_p(s.cuda_stream))
    if rc != SCONV_OK:
        raise SconvError(rc, f"sconv_fc_tune (hip error {lib().sconv_last_hip_error(csr.handle)})")
    return out_t


def sconv_machine_gfx950() -> sconv_machine:
    m = sconv_machine()
    lib().sconv_machine_gfx950(C.byref(m))
    return m


def sconv_model_predict(layer, N: int, density: float, csr: Csr | None = None, machine: sconv_machine | None = None):
    d = make_desc(layer)
    p = sconv_prediction()
    _check(lib().sconv_model_predict(C.byref(d), N, float(density), csr.handle if csr else None,
                                     C.byref(machine) if machine is not None else None, C.byref(p)),
           "sconv_model_predict")
    return p.as_dict()


def sconv_model_predict_lowered(layer, N: int, density: float, csr: Csr | None = None, machine: sconv_machine | None = None):
    d = make_desc(layer)
    p = sconv_prediction()
    _check(lib().sconv_model_predict_lowered(C.byref(d), N, float(density), csr.handle if csr else None,
                                             C.byref(machine) if machine is not None else None, C.byref(p)),
           "sconv_model_predict_lowered")
    return p.as_dict()


def sconv_lower_offsets(layer, layout: int, rowptr, colidx):
    """(off int32[nnz], step_y, step_x) for a padded image stored in `layout` (LAYOUT_CHW or LAYOUT_HWC)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    d = make_desc(layer)
    off = np.zeros(max(len(colidx), 1), dtype=np.int32)
    sy, sx = C.c_int32(), C.c_int32()
    _check(lib().sconv_lower_offsets(C.byref(d), int(layout), _np_ptr(rowptr), _np_ptr(colidx), _np_ptr(off),
                                     C.byref(sy), C.byref(sx)), "sconv_lower_offsets")
    return off[:len(colidx)], sy.value, sx.value


def sconv_csr_balance(h) -> dict:
    """Load-balance figures of the kernel-3 packing (stream chunks of 8 entries)."""
    b = sconv_balance()
    _check(lib().sconv_csr_balance(h.handle, C.byref(b)), "sconv_csr_balance")
    return {n: getattr(b, n) for n, _ in sconv_balance._fields_}


def sconv_gsl_decide(layer, N: int, density: float, stabilized: bool = False, machine: sconv_machine | None = None):
    """(action name, prediction dict) of the pruning controller for one layer."""
    d = make_desc(layer)
    act = C.c_int32(-1)
    p = sconv_prediction()
    _check(lib().sconv_gsl_decide(C.byref(d), N, float(density), int(bool(stabilized)),
                                  C.byref(machine) if machine is not None else None, C.byref(act), C.byref(p)),
           "sconv_gsl_decide")
    return GSL_ACTIONS[act.value], p.as_dict()
