"""CPU oracle for the SOAR hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes view of ``soar_oracle.c`` (built by ``oracle/build.py`` into
``oracle/libsoar_oracle.so``).  Nothing in the product package imports this
module; it is used by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  It shares no code with the HIP path.

Arrays are numpy; bf16 weights travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

BF16, FP32 = 0, 1
METHOD_RTN, METHOD_SOAR = 0, 1
STATUS_NONFINITE, STATUS_ALLZERO, STATUS_BAD_AMAX = 1, 2, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
# SOAR_ORACLE_LIB lets the mutation test point the pins at a deliberately broken build
_LIB_PATH = os.environ.get("SOAR_ORACLE_LIB") or os.path.join(_HERE, "libsoar_oracle.so")
_lib = None


class _Trace(C.Structure):
    _fields_ = [
        ("alpha0", C.c_float), ("alpha1", C.c_float),
        ("N", C.c_double), ("M", C.c_double),
        ("code0", C.c_void_p), ("nib0", C.c_void_p),
        ("a", C.c_void_p), ("b", C.c_void_p),
        ("delta_star", C.c_void_p), ("centre", C.c_void_p),
        ("err_best", C.c_void_p),
    ]


class _IterParams(C.Structure):
    _fields_ = [("iters", C.c_int32), ("n_beta", C.c_int32), ("beta_lo", C.c_float), ("beta_hi", C.c_float),
                ("dd_mode", C.c_int32), ("dss_radius", C.c_int32), ("early_stop_rel", C.c_float),
                ("arm", C.c_int32)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        L = C.CDLL(_LIB_PATH)
        L.soar_oracle_bf16_to_f32.restype = C.c_float
        L.soar_oracle_bf16_to_f32.argtypes = [C.c_uint16]
        L.soar_oracle_f32_to_bf16.restype = C.c_uint16
        L.soar_oracle_f32_to_bf16.argtypes = [C.c_float]
        L.soar_oracle_e2m1_round.restype = C.c_float
        L.soar_oracle_e2m1_round.argtypes = [C.c_float]
        L.soar_oracle_e2m1_nibble.restype = C.c_uint8
        L.soar_oracle_e2m1_nibble.argtypes = [C.c_float]
        L.soar_oracle_e2m1_value.restype = C.c_float
        L.soar_oracle_e2m1_value.argtypes = [C.c_uint8]
        L.soar_oracle_e4m3_value.restype = C.c_float
        L.soar_oracle_e4m3_value.argtypes = [C.c_uint8]
        L.soar_oracle_e4m3_project.restype = C.c_uint8
        L.soar_oracle_e4m3_project.argtypes = [C.c_float]
        L.soar_oracle_quantize.restype = C.c_int
        L.soar_oracle_quantize.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int,
            C.c_void_p, C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_double),
            C.POINTER(C.c_int32), C.POINTER(_Trace)]
        L.soar_oracle_quantize_iter.restype = C.c_int
        L.soar_oracle_quantize_iter.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.POINTER(_IterParams),
            C.c_void_p, C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_double),
            C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
        L.soar_oracle_quantize_rtn_amax.restype = C.c_int
        L.soar_oracle_quantize_rtn_amax.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_float,
            C.c_void_p, C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        L.soar_oracle_mxfp4_quantize.restype = C.c_int
        L.soar_oracle_mxfp4_quantize.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int32, C.c_float, C.c_float,
            C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        L.soar_oracle_mxfp4_dequantize.restype = C.c_int
        L.soar_oracle_mxfp4_dequantize.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_int64]
        L.soar_oracle_dequantize.restype = C.c_int
        L.soar_oracle_dequantize.argtypes = [
            C.c_void_p, C.c_void_p, C.c_float, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_int64]
        L.soar_oracle_recon_error.restype = C.c_int
        L.soar_oracle_recon_error.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_float, C.POINTER(C.c_double)]
        L.soar_oracle_threads.restype = C.c_int
        L.soar_oracle_set_threads.argtypes = [C.c_int]
        L.soar_oracle_e2m1_nibble_many.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.soar_oracle_e4m3_project_many.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        _lib = L
    return _lib


# ---------------------------------------------------------------- primitives
def e2m1_round(x: float) -> float:
    return float(lib().soar_oracle_e2m1_round(C.c_float(x)))


def e2m1_nibble(x: float) -> int:
    return int(lib().soar_oracle_e2m1_nibble(C.c_float(x)))


def e2m1_value(nibble: int) -> float:
    return float(lib().soar_oracle_e2m1_value(C.c_uint8(nibble)))


def e4m3_value(code: int) -> float:
    return float(lib().soar_oracle_e4m3_value(C.c_uint8(code)))


def e4m3_project(y: float) -> int:
    return int(lib().soar_oracle_e4m3_project(C.c_float(y)))


def e2m1_nibble_many(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().soar_oracle_e2m1_nibble_many(x.ctypes.data, x.size, out.ctypes.data)
    return out


def e4m3_project_many(y: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float32)
    out = np.empty(y.shape, dtype=np.uint8)
    lib().soar_oracle_e4m3_project_many(y.ctypes.data, y.size, out.ctypes.data)
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(x: float) -> int:
    return int(lib().soar_oracle_f32_to_bf16(C.c_float(x)))


def threads() -> int:
    return int(lib().soar_oracle_threads())


def set_threads(n: int) -> None:
    lib().soar_oracle_set_threads(int(n))


# ---------------------------------------------------------------- whole path
@dataclass
class Quantized:
    codes: np.ndarray          # uint8 [rows, cols/2]
    scales: np.ndarray         # uint8 [rows, cols/16]
    global_scale: float        # value of the float32 global scale
    sse: float
    status: int
    trace: Optional[dict] = None


def _dtype_of(w: np.ndarray) -> int:
    if w.dtype == np.uint16:
        return BF16
    if w.dtype == np.float32:
        return FP32
    raise TypeError("weights must be uint16 (bf16 bits) or float32")


def _check2d(w: np.ndarray):
    if w.ndim != 2:
        raise ValueError("weights must be 2-D")
    if w.strides[1] != w.itemsize or w.strides[0] % w.itemsize:
        raise ValueError("rows must be contiguous")
    return w.shape[0], w.shape[1], w.strides[0] // w.itemsize


def quantize(w: np.ndarray, method: int = METHOD_SOAR, dss_radius: int = 4,
             want_trace: bool = False) -> Quantized:
    rows, cols, ld = _check2d(w)
    dt = _dtype_of(w)
    nblk = rows * (cols // 16)
    codes = np.zeros((rows, cols // 2), dtype=np.uint8)
    scales = np.zeros((rows, cols // 16), dtype=np.uint8)
    g = C.c_float(0.0)
    sse = C.c_double(0.0)
    st = C.c_int32(0)
    tr = None
    bufs = None
    if want_trace:
        bufs = dict(
            code0=np.zeros(nblk, np.uint8), nib0=np.zeros(nblk * 8, np.uint8),
            a=np.zeros(nblk, np.float32), b=np.zeros(nblk, np.float32),
            delta_star=np.zeros(nblk, np.float32), centre=np.zeros(nblk, np.uint8),
            err_best=np.zeros(nblk, np.float32))
        tr = _Trace()
        for k, v in bufs.items():
            setattr(tr, k, v.ctypes.data)
    rc = lib().soar_oracle_quantize(
        w.ctypes.data, dt, rows, cols, ld, method, dss_radius,
        codes.ctypes.data, scales.ctypes.data, C.byref(g), C.byref(sse), C.byref(st),
        C.byref(tr) if tr is not None else None)
    if rc != 0:
        raise ValueError("soar_oracle_quantize: bad argument")
    trace = None
    if want_trace:
        trace = dict(bufs)
        trace.update(alpha0=np.float32(tr.alpha0), alpha1=np.float32(tr.alpha1), N=tr.N, M=tr.M)
    return Quantized(codes, scales, np.float32(g.value), float(sse.value), int(st.value), trace)


def quantize_rtn_amax(w: np.ndarray, amax: float) -> Quantized:
    """Max-based NVFP4 (Sec. 3.1) with a supplied tensor maximum."""
    rows, cols, ld = _check2d(w)
    codes = np.zeros((rows, cols // 2), dtype=np.uint8)
    scales = np.zeros((rows, cols // 16), dtype=np.uint8)
    g = C.c_float(0.0)
    sse = C.c_double(0.0)
    st = C.c_int32(0)
    rc = lib().soar_oracle_quantize_rtn_amax(w.ctypes.data, _dtype_of(w), rows, cols, ld, C.c_float(amax),
                                             codes.ctypes.data, scales.ctypes.data, C.byref(g), C.byref(sse),
                                             C.byref(st))
    if rc != 0:
        raise ValueError("soar_oracle_quantize_rtn_amax: bad argument")
    return Quantized(codes, scales, np.float32(g.value), float(sse.value), int(st.value), None)


def mxfp4_quantize(w: np.ndarray, dss: bool = False, n_beta: int = 101, beta_lo: float = 0.5,
                   beta_hi: float = 1.5, radius: int = 1) -> Quantized:
    """MXFP4 (blocks of 32, E8M0 scale bytes), plain or with the decoupled scale search.
    The returned global_scale is 1 (the format has none)."""
    rows, cols, ld = _check2d(w)
    codes = np.zeros((rows, cols // 2), dtype=np.uint8)
    scales = np.zeros((rows, cols // 32), dtype=np.uint8)
    sse, st = C.c_double(0.0), C.c_int32(0)
    rc = lib().soar_oracle_mxfp4_quantize(w.ctypes.data, _dtype_of(w), rows, cols, ld, 1 if dss else 0, n_beta,
                                          beta_lo, beta_hi, radius, codes.ctypes.data, scales.ctypes.data,
                                          C.byref(sse), C.byref(st))
    if rc != 0:
        raise ValueError("soar_oracle_mxfp4_quantize: bad argument")
    return Quantized(codes, scales, np.float32(1.0), float(sse.value), int(st.value), None)


def mxfp4_dequantize(codes: np.ndarray, scales: np.ndarray, out_dtype: int = FP32) -> np.ndarray:
    rows, cols = scales.shape[0], scales.shape[1] * 32
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    out = np.zeros((rows, cols), dtype=np.uint16 if out_dtype == BF16 else np.float32)
    rc = lib().soar_oracle_mxfp4_dequantize(codes.ctypes.data, scales.ctypes.data, rows, cols, out_dtype,
                                            out.ctypes.data, cols)
    if rc != 0:
        raise ValueError("soar_oracle_mxfp4_dequantize: bad argument")
    return out


DD_WINDOW, DD_BRACKET = 0, 1
ARM_SOAR, ARM_CJSO_ONLY, ARM_DSS_ONLY = 0, 1, 2


def quantize_iter(w: np.ndarray, iters: int = 15, n_beta: int = 101, beta_lo: float = 0.5,
                  beta_hi: float = 1.5, dd_mode: int = DD_BRACKET, dss_radius: int = 1,
                  early_stop_rel: float = 1e-3, arm: int = 0) -> Quantized:
    """Algorithm 1 in full (defaults: the paper's settings).  The returned trace holds
    ``sse_trace`` (error of the Eq. 1-2 state, then after every iteration run) and
    ``iters_run``.  arm: ARM_SOAR, ARM_CJSO_ONLY or ARM_DSS_ONLY (the ablation arms)."""
    rows, cols, ld = _check2d(w)
    dt = _dtype_of(w)
    codes = np.zeros((rows, cols // 2), dtype=np.uint8)
    scales = np.zeros((rows, cols // 16), dtype=np.uint8)
    g, sse, st, it = C.c_float(0.0), C.c_double(0.0), C.c_int32(0), C.c_int32(0)
    tracebuf = np.full(iters + 1, np.nan, dtype=np.float64)
    p = _IterParams(iters, n_beta, beta_lo, beta_hi, dd_mode, dss_radius, early_stop_rel, arm)
    rc = lib().soar_oracle_quantize_iter(w.ctypes.data, dt, rows, cols, ld, C.byref(p), codes.ctypes.data,
                                         scales.ctypes.data, C.byref(g), C.byref(sse), C.byref(st),
                                         C.byref(it), tracebuf.ctypes.data)
    if rc != 0:
        raise ValueError("soar_oracle_quantize_iter: bad argument")
    return Quantized(codes, scales, np.float32(g.value), float(sse.value), int(st.value),
                     dict(sse_trace=tracebuf, iters_run=int(it.value)))


def dequantize(codes: np.ndarray, scales: np.ndarray, global_scale, out_dtype: int = FP32) -> np.ndarray:
    rows, cols = scales.shape[0], scales.shape[1] * 16
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    out = np.zeros((rows, cols), dtype=np.uint16 if out_dtype == BF16 else np.float32)
    rc = lib().soar_oracle_dequantize(codes.ctypes.data, scales.ctypes.data,
                                      C.c_float(float(global_scale)), rows, cols, out_dtype,
                                      out.ctypes.data, cols)
    if rc != 0:
        raise ValueError("soar_oracle_dequantize: bad argument")
    return out


def recon_error(w: np.ndarray, codes: np.ndarray, scales: np.ndarray, global_scale) -> float:
    rows, cols, ld = _check2d(w)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    sse = C.c_double(0.0)
    rc = lib().soar_oracle_recon_error(w.ctypes.data, _dtype_of(w), rows, cols, ld,
                                       codes.ctypes.data, scales.ctypes.data,
                                       C.c_float(float(global_scale)), C.byref(sse))
    if rc != 0:
        raise ValueError("soar_oracle_recon_error: bad argument")
    return float(sse.value)
