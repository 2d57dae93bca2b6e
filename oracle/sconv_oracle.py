"""ctypes face of the CPU oracle (sconv_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this.  It neither imports nor is imported by the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sconv_oracle.c")
_LIB = os.path.join(_HERE, "libsconv_oracle.so")
_lib = None


class Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("C", "H", "W", "K", "R", "S", "stride", "pad", "groups")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP for the timed variant)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_csr_from_dense.restype = C.c_int64
        L.oracle_csr_from_dense.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_lower_offsets.restype = C.c_int
        L.oracle_lower_offsets.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_lower_offsets_hwc.restype = C.c_int
        L.oracle_lower_offsets_hwc.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_forward_f64.restype = C.c_int
        L.oracle_forward_f64.argtypes = [C.POINTER(Desc), C.c_int32] + [C.c_void_p] * 6
        L.oracle_forward_f32.restype = C.c_int
        L.oracle_forward_f32.argtypes = [C.POINTER(Desc), C.c_int32] + [C.c_void_p] * 5 + [C.c_int]
        L.oracle_out_h.argtypes = [C.POINTER(Desc)]
        L.oracle_out_w.argtypes = [C.POINTER(Desc)]
        _lib = L
    return _lib


def _desc(layer) -> Desc:
    return Desc(*(int(getattr(layer, n)) for n in ("C", "H", "W", "K", "R", "S", "stride", "pad", "groups")))


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def out_hw(layer):
    d = _desc(layer)
    L = _load()
    return L.oracle_out_h(C.byref(d)), L.oracle_out_w(C.byref(d))


def csr_from_dense(layer, w: np.ndarray):
    """Dense [K][C/groups][R][S] fp32 -> (rowptr int32[K+1], colidx int32[nnz], val fp32[nnz])."""
    L = _load()
    d = _desc(layer)
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.shape == (layer.K, layer.C // layer.groups, layer.R, layer.S)
    nnz = L.oracle_csr_from_dense(C.byref(d), _p(w), None, None, None)
    if nnz < 0:
        raise ValueError("bad descriptor")
    rowptr = np.zeros(layer.K + 1, dtype=np.int32)
    colidx = np.zeros(nnz, dtype=np.int32)
    val = np.zeros(nnz, dtype=np.float32)
    L.oracle_csr_from_dense(C.byref(d), _p(w), _p(rowptr), _p(colidx), _p(val))
    return rowptr, colidx, val


def lower_offsets(layer, rowptr, colidx):
    """Column indices -> offsets into the zero-padded CHW image (Figure 2's f)."""
    L = _load()
    d = _desc(layer)
    off = np.zeros(len(colidx), dtype=np.int32)
    rc = L.oracle_lower_offsets(C.byref(d), _p(rowptr), _p(colidx), _p(off))
    if rc:
        raise ValueError(f"oracle_lower_offsets failed: {rc}")
    return off


def lower_offsets_hwc(layer, rowptr, colidx):
    """Column indices -> offsets into the zero-padded HWC image (channel innermost)."""
    L = _load()
    d = _desc(layer)
    off = np.zeros(len(colidx), dtype=np.int32)
    rc = L.oracle_lower_offsets_hwc(C.byref(d), _p(rowptr), _p(colidx), _p(off))
    if rc:
        raise ValueError(f"oracle_lower_offsets_hwc failed: {rc}")
    return off


def forward_f64(layer, rowptr, off, val, x: np.ndarray, want_absum: bool = True):
    """fp64 sums and sums of |products|, each [N][K][OH][OW]."""
    L = _load()
    d = _desc(layer)
    x = np.ascontiguousarray(x, dtype=np.float32)
    N = x.shape[0]
    OH, OW = out_hw(layer)
    out = np.zeros((N, layer.K, OH, OW), dtype=np.float64)
    ab = np.zeros_like(out) if want_absum else None
    rc = L.oracle_forward_f64(C.byref(d), N, _p(rowptr), _p(off), _p(val), _p(x), _p(out), _p(ab))
    if rc:
        raise RuntimeError(f"oracle_forward_f64 failed: {rc}")
    return out, ab


def forward_f32(layer, rowptr, off, val, x: np.ndarray, nthreads: int = 0):
    """Figure 2 in fp32, CSR order.  Returns (out fp32, threads used)."""
    L = _load()
    d = _desc(layer)
    x = np.ascontiguousarray(x, dtype=np.float32)
    N = x.shape[0]
    OH, OW = out_hw(layer)
    out = np.empty((N, layer.K, OH, OW), dtype=np.float32)
    rc = L.oracle_forward_f32(C.byref(d), N, _p(rowptr), _p(off), _p(val), _p(x), _p(out), nthreads)
    if rc < 0:
        raise RuntimeError(f"oracle_forward_f32 failed: {rc}")
    return out, rc


def sparse_conv(layer, w: np.ndarray, x: np.ndarray):
    """Convenience: dense-shaped pruned weights -> (fp64 out, fp64 absum, csr tuple)."""
    rowptr, colidx, val = csr_from_dense(layer, w)
    off = lower_offsets(layer, rowptr, colidx)
    out, ab = forward_f64(layer, rowptr, off, val, x)
    return out, ab, (rowptr, colidx, off, val)


def bias_relu(out: np.ndarray, absum: np.ndarray, bias, relu: bool):
    """Epilogue applied to a convolution result [N][K][OH][OW] in fp64: out + bias[k], then max(., 0).
    (Not in the paper; the plain definition of the bias and ReLU layers that follow a convolution.)
    Returns (result, scale): scale = absum + |bias[k]| is the sum of the magnitudes of everything added
    into an output, the yardstick of the fp32 tolerance."""
    res = np.array(out, dtype=np.float64, copy=True)
    scale = np.array(absum, dtype=np.float64, copy=True)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64).reshape(1, -1, 1, 1)
        res += b
        scale += np.abs(b)
    if relu:
        res = np.where(res > 0, res, 0.0)
    return res, scale
