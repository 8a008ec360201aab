"""ctypes view of the HIP library's C-ABI (``include/soar.h``).

Argument marshalling only: every step of the method runs inside the HIP
kernels.  torch is used for device memory and streams.  There is no CPU
fallback -- if ``libsoar_hip.so`` has not been built, or no GPU is present,
the entry points raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

SOAR_OK = 0
SOAR_ERR_TOO_LARGE = 8
SOAR_STATIC_MAX_BLOCKS = 1 << 22
SOAR_BF16, SOAR_FP32 = 0, 1
SOAR_METHOD_RTN, SOAR_METHOD_SOAR, SOAR_METHOD_CJSO_ONLY, SOAR_METHOD_DSS_ONLY = 0, 1, 2, 3
SOAR_SEARCH_AUTO, SOAR_SEARCH_FULL = 0, 1
SOAR_STATUS_NONFINITE, SOAR_STATUS_ALLZERO, SOAR_STATUS_BAD_AMAX, SOAR_STATUS_GAVE_UP = 1, 2, 4, 8
SOAR_RESIDENT_AUTO, SOAR_RESIDENT_NEVER = 0, 1
SOAR_DD_WINDOW, SOAR_DD_BRACKET = 0, 1
(SOAR_KERNEL_INIT, SOAR_KERNEL_ABSMAX, SOAR_KERNEL_STATS, SOAR_KERNEL_SEARCH,
 SOAR_KERNEL_DEQUANT, SOAR_KERNEL_RECON, SOAR_KERNEL_ITER_INIT, SOAR_KERNEL_ITER, SOAR_KERNEL_MX,
 SOAR_KERNEL_RESIDENT, SOAR_KERNEL_COUNT) = range(11)

EXPORTS = (
    "soar_default_params", "soar_paper_params", "soar_workspace_bytes", "soar_batch_workspace_bytes", "soar_quantize",
    "soar_quantize_batch", "soar_quantize_static",
    "soar_dequantize", "soar_recon_error", "soar_dequantize_batch", "soar_recon_error_batch",
    "soar_e2m1_round_f32", "soar_e4m3_project_f32",
    "soar_rcp_midrange_f32",
    "soar_mx_default_params", "soar_mxfp4_workspace_bytes", "soar_mxfp4_quantize", "soar_mxfp4_dequantize",
    "soar_mxfp4_dequantize_batch",
    "soar_mxfp4_quantize_batch", "soar_mxfp4_batch_workspace_bytes",
    "soar_kernel_timing_enable", "soar_kernel_timing_read", "soar_search_stats_enable", "soar_search_stats_read",
    "soar_debug_arrival_plan", "soar_status_string", "soar_version",
)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsoar_hip.so")
_lib = None


class SoarError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().soar_status_string(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (status {code})")


class soar_params(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("method", C.c_int32), ("block", C.c_int32),
        ("iters", C.c_int32), ("dss_radius", C.c_int32), ("n_beta", C.c_int32),
        ("beta_lo", C.c_float), ("beta_hi", C.c_float), ("early_stop_rel", C.c_float),
        ("search_mode", C.c_int32), ("tiles_per_wg", C.c_int32), ("streams", C.c_int32),
        ("dd_mode", C.c_int32), ("resident", C.c_int32), ("resident_wait_us", C.c_int32),
        ("tiles_per_wg_absmax", C.c_int32), ("tiles_per_wg_search", C.c_int32),
    ]


class soar_mx_params(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dss", C.c_int32), ("n_beta", C.c_int32), ("beta_lo", C.c_float),
        ("beta_hi", C.c_float), ("radius", C.c_int32), ("tiles_per_wg", C.c_int32), ("single_pass", C.c_int32),
        ("streams", C.c_int32),
    ]


class soar_stored_desc(C.Structure):
    _fields_ = [
        ("d_codes", C.c_void_p), ("d_scales", C.c_void_p), ("d_global_scale", C.c_void_p),
        ("rows", C.c_int64), ("cols", C.c_int64), ("ld_elems", C.c_int64),
        ("dtype", C.c_int32), ("reserved", C.c_int32),
        ("d_w", C.c_void_p), ("d_out", C.c_void_p), ("d_sse", C.c_void_p),
    ]


class soar_mx_tensor_desc(C.Structure):
    _fields_ = [
        ("d_w", C.c_void_p), ("dtype", C.c_int32),
        ("rows", C.c_int64), ("cols", C.c_int64), ("ld_elems", C.c_int64),
        ("d_codes", C.c_void_p), ("d_scales", C.c_void_p), ("d_sse", C.c_void_p), ("d_status", C.c_void_p),
    ]


class soar_tensor_desc(C.Structure):
    _fields_ = [
        ("d_w", C.c_void_p), ("dtype", C.c_int32),
        ("rows", C.c_int64), ("cols", C.c_int64), ("ld_elems", C.c_int64),
        ("d_codes", C.c_void_p), ("d_scales", C.c_void_p), ("d_global_scale", C.c_void_p),
        ("d_sse", C.c_void_p), ("d_status", C.c_void_p),
        ("d_iters_run", C.c_void_p), ("d_sse_trace", C.c_void_p), ("d_amax_in", C.c_void_p),
    ]


def lib():
    """Load the HIP library; raise loudly when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it with `python -m paper_2605_12245_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    L.soar_default_params.argtypes = [C.POINTER(soar_params)]
    L.soar_default_params.restype = None
    L.soar_paper_params.argtypes = [C.POINTER(soar_params)]
    L.soar_paper_params.restype = None
    L.soar_workspace_bytes.argtypes = [i64, i64, C.POINTER(soar_params)]
    L.soar_workspace_bytes.restype = C.c_size_t
    L.soar_batch_workspace_bytes.argtypes = [i32, C.POINTER(soar_tensor_desc), C.POINTER(soar_params)]
    L.soar_batch_workspace_bytes.restype = C.c_size_t
    L.soar_quantize.argtypes = [vp, i32, i64, i64, i64, C.POINTER(soar_params), vp, vp, vp, vp, vp,
                                vp, C.c_size_t, vp]
    L.soar_quantize.restype = i32
    L.soar_quantize_static.argtypes = [vp, i32, i64, i64, i64, C.POINTER(soar_params), vp, vp, vp, vp, vp, vp]
    L.soar_quantize_static.restype = i32
    L.soar_quantize_batch.argtypes = [i32, C.POINTER(soar_tensor_desc), C.POINTER(soar_params), vp,
                                      C.c_size_t, vp]
    L.soar_quantize_batch.restype = i32
    L.soar_dequantize.argtypes = [vp, vp, vp, i64, i64, i32, vp, i64, vp]
    L.soar_dequantize.restype = i32
    L.soar_recon_error.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, vp, vp]
    L.soar_recon_error.restype = i32
    L.soar_dequantize_batch.argtypes = [i32, C.POINTER(soar_stored_desc), vp]
    L.soar_dequantize_batch.restype = i32
    L.soar_recon_error_batch.argtypes = [i32, C.POINTER(soar_stored_desc), vp]
    L.soar_recon_error_batch.restype = i32
    L.soar_e2m1_round_f32.argtypes = [vp, i64, vp, vp]
    L.soar_e2m1_round_f32.restype = i32
    L.soar_e4m3_project_f32.argtypes = [vp, i64, vp, vp]
    L.soar_e4m3_project_f32.restype = i32
    L.soar_mx_default_params.argtypes = [C.POINTER(soar_mx_params)]
    L.soar_mx_default_params.restype = None
    L.soar_mxfp4_workspace_bytes.argtypes = [i64, i64, C.POINTER(soar_mx_params)]
    L.soar_mxfp4_workspace_bytes.restype = C.c_size_t
    L.soar_mxfp4_quantize.argtypes = [vp, i32, i64, i64, i64, C.POINTER(soar_mx_params), vp, vp, vp, vp, vp,
                                      C.c_size_t, vp]
    L.soar_mxfp4_quantize.restype = i32
    L.soar_mxfp4_quantize_batch.argtypes = [i32, C.POINTER(soar_mx_tensor_desc), C.POINTER(soar_mx_params), vp,
                                            C.c_size_t, vp]
    L.soar_mxfp4_quantize_batch.restype = i32
    L.soar_mxfp4_batch_workspace_bytes.argtypes = [i32, C.POINTER(soar_mx_tensor_desc), C.POINTER(soar_mx_params)]
    L.soar_mxfp4_batch_workspace_bytes.restype = C.c_size_t
    L.soar_mxfp4_dequantize.argtypes = [vp, vp, i64, i64, i32, vp, i64, vp]
    L.soar_mxfp4_dequantize.restype = i32
    L.soar_mxfp4_dequantize_batch.argtypes = [i32, C.POINTER(soar_stored_desc), vp]
    L.soar_mxfp4_dequantize_batch.restype = i32
    L.soar_rcp_midrange_f32.argtypes = [vp, i64, vp, vp]
    L.soar_rcp_midrange_f32.restype = i32
    L.soar_kernel_timing_enable.argtypes = [C.c_int]
    L.soar_kernel_timing_enable.restype = None
    L.soar_kernel_timing_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
    L.soar_kernel_timing_read.restype = i32
    L.soar_search_stats_enable.argtypes = [C.c_int]
    L.soar_search_stats_enable.restype = i32
    L.soar_search_stats_read.argtypes = [C.POINTER(i64)]
    L.soar_search_stats_read.restype = i32
    L.soar_debug_arrival_plan.argtypes = [C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32)]
    L.soar_debug_arrival_plan.restype = None
    L.soar_status_string.argtypes = [i32]
    L.soar_status_string.restype = C.c_char_p
    L.soar_version.argtypes = []
    L.soar_version.restype = C.c_uint32
    _lib = L
    return L


# ------------------------------------------------------------------ raw entry points
def soar_default_params(method: int = SOAR_METHOD_SOAR, dss_radius: int = 4,
                        search_mode: int = SOAR_SEARCH_AUTO, tiles_per_wg: int = 0,
                        streams: int = 0) -> soar_params:
    p = soar_params()
    lib().soar_default_params(C.byref(p))
    p.method = method
    p.dss_radius = dss_radius
    p.search_mode = search_mode
    p.tiles_per_wg = tiles_per_wg
    p.streams = streams
    return p


def soar_paper_params(iters: Optional[int] = None, n_beta: Optional[int] = None,
                      beta_lo: Optional[float] = None, beta_hi: Optional[float] = None,
                      dd_mode: Optional[int] = None, dss_radius: Optional[int] = None,
                      early_stop_rel: Optional[float] = None, tiles_per_wg: int = 0,
                      streams: int = 0) -> soar_params:
    """The full algorithm's settings; any argument given overrides one field."""
    p = soar_params()
    lib().soar_paper_params(C.byref(p))
    for name, v in (("iters", iters), ("n_beta", n_beta), ("beta_lo", beta_lo), ("beta_hi", beta_hi),
                    ("dd_mode", dd_mode), ("dss_radius", dss_radius), ("early_stop_rel", early_stop_rel)):
        if v is not None:
            setattr(p, name, v)
    p.tiles_per_wg = tiles_per_wg
    p.streams = streams
    return p


def soar_arm_params(method: int, iters: int = 15, early_stop_rel: float = 1e-3, n_beta: int = 101,
                    beta_lo: float = 0.5, beta_hi: float = 1.5, dss_radius: int = 1, tiles_per_wg: int = 0,
                    streams: int = 0) -> soar_params:
    """Settings for one arm of the component study: SOAR_METHOD_CJSO_ONLY (takes no search settings)
    or SOAR_METHOD_DSS_ONLY (window candidates of the given radius, beta grid)."""
    p = soar_params()
    lib().soar_default_params(C.byref(p))
    p.method = method
    p.iters = iters
    p.early_stop_rel = early_stop_rel
    p.tiles_per_wg = tiles_per_wg
    p.streams = streams
    if method == SOAR_METHOD_CJSO_ONLY:
        p.dss_radius = 0
    else:
        p.n_beta, p.beta_lo, p.beta_hi, p.dss_radius = n_beta, beta_lo, beta_hi, dss_radius
    return p


def soar_workspace_bytes(rows: int, cols: int, params: soar_params) -> int:
    return int(lib().soar_workspace_bytes(rows, cols, C.byref(params)))


def soar_batch_workspace_bytes(descs: Sequence[soar_tensor_desc], params: soar_params) -> int:
    arr = (soar_tensor_desc * len(descs))(*descs)
    return int(lib().soar_batch_workspace_bytes(len(descs), arr, C.byref(params)))


def soar_quantize(d_w, dtype, rows, cols, ld_elems, params, d_codes, d_scales, d_global_scale,
                  d_sse, d_status, d_workspace, workspace_bytes, hip_stream) -> int:
    """Raw call: device addresses as integers; returns the soar_status code."""
    return int(lib().soar_quantize(d_w, dtype, rows, cols, ld_elems, C.byref(params), d_codes, d_scales,
                                   d_global_scale, d_sse, d_status, d_workspace, workspace_bytes,
                                   hip_stream))


def soar_quantize_static(d_w, dtype, rows, cols, ld_elems, params, d_codes, d_scales, d_global_scale,
                         d_sse, d_status, hip_stream) -> int:
    """Raw call of the entry point that uses the library's built-in workspace."""
    return int(lib().soar_quantize_static(d_w, dtype, rows, cols, ld_elems, C.byref(params), d_codes, d_scales,
                                          d_global_scale, d_sse, d_status, hip_stream))


def soar_quantize_batch(descs: Sequence[soar_tensor_desc], params, d_workspace, workspace_bytes,
                        hip_stream) -> int:
    arr = (soar_tensor_desc * len(descs))(*descs)
    return int(lib().soar_quantize_batch(len(descs), arr, C.byref(params), d_workspace, workspace_bytes,
                                         hip_stream))


def soar_dequantize(d_codes, d_scales, d_global_scale, rows, cols, out_dtype, d_out, ld_elems,
                    hip_stream) -> int:
    return int(lib().soar_dequantize(d_codes, d_scales, d_global_scale, rows, cols, out_dtype, d_out,
                                     ld_elems, hip_stream))


def soar_recon_error(d_w, dtype, rows, cols, ld_elems, d_codes, d_scales, d_global_scale, d_sse,
                     hip_stream) -> int:
    return int(lib().soar_recon_error(d_w, dtype, rows, cols, ld_elems, d_codes, d_scales,
                                      d_global_scale, d_sse, hip_stream))


def soar_e2m1_round_f32(d_x, n, d_out, hip_stream) -> int:
    return int(lib().soar_e2m1_round_f32(d_x, n, d_out, hip_stream))


def soar_e4m3_project_f32(d_x, n, d_out, hip_stream) -> int:
    return int(lib().soar_e4m3_project_f32(d_x, n, d_out, hip_stream))


def soar_mx_default_params(dss: bool = True, n_beta: Optional[int] = None, beta_lo: Optional[float] = None,
                           beta_hi: Optional[float] = None, radius: Optional[int] = None,
                           tiles_per_wg: int = 0, single_pass: bool = False, streams: int = 0) -> soar_mx_params:
    p = soar_mx_params()
    lib().soar_mx_default_params(C.byref(p))
    p.dss = 1 if dss else 0
    for name, v in (("n_beta", n_beta), ("beta_lo", beta_lo), ("beta_hi", beta_hi), ("radius", radius)):
        if v is not None:
            setattr(p, name, v)
    p.tiles_per_wg = tiles_per_wg
    p.single_pass = 1 if single_pass else 0
    p.streams = streams
    return p


def soar_mxfp4_workspace_bytes(rows: int, cols: int, params: soar_mx_params) -> int:
    return int(lib().soar_mxfp4_workspace_bytes(rows, cols, C.byref(params)))


def soar_mxfp4_quantize(d_w, dtype, rows, cols, ld_elems, params, d_codes, d_scales, d_sse, d_status,
                        d_workspace, workspace_bytes, hip_stream) -> int:
    return int(lib().soar_mxfp4_quantize(d_w, dtype, rows, cols, ld_elems, C.byref(params), d_codes, d_scales,
                                         d_sse, d_status, d_workspace, workspace_bytes, hip_stream))


def soar_mxfp4_quantize_batch(descs: Sequence[soar_mx_tensor_desc], params, d_workspace, workspace_bytes,
                              hip_stream) -> int:
    arr = (soar_mx_tensor_desc * len(descs))(*descs)
    return int(lib().soar_mxfp4_quantize_batch(len(descs), arr, C.byref(params), d_workspace, workspace_bytes,
                                               hip_stream))


def soar_mxfp4_batch_workspace_bytes(descs: Sequence[soar_mx_tensor_desc], params) -> int:
    arr = (soar_mx_tensor_desc * len(descs))(*descs)
    return int(lib().soar_mxfp4_batch_workspace_bytes(len(descs), arr, C.byref(params)))


def _stored_array(descs):
    arr = (soar_stored_desc * max(1, len(descs)))()
    for k, d in enumerate(descs):
        arr[k] = d
    return arr


def soar_dequantize_batch(descs: Sequence["soar_stored_desc"], hip_stream) -> int:
    return int(lib().soar_dequantize_batch(len(descs), _stored_array(descs), hip_stream))


def soar_recon_error_batch(descs: Sequence["soar_stored_desc"], hip_stream) -> int:
    return int(lib().soar_recon_error_batch(len(descs), _stored_array(descs), hip_stream))


def soar_mxfp4_dequantize(d_codes, d_scales, rows, cols, out_dtype, d_out, ld_elems, hip_stream) -> int:
    return int(lib().soar_mxfp4_dequantize(d_codes, d_scales, rows, cols, out_dtype, d_out, ld_elems, hip_stream))


def soar_mxfp4_dequantize_batch(descs: Sequence["soar_stored_desc"], hip_stream) -> int:
    return int(lib().soar_mxfp4_dequantize_batch(len(descs), _stored_array(descs), hip_stream))


def soar_rcp_midrange_f32(d_x, n, d_out, hip_stream) -> int:
    return int(lib().soar_rcp_midrange_f32(d_x, n, d_out, hip_stream))


def soar_kernel_timing_enable(enable: bool) -> None:
    lib().soar_kernel_timing_enable(1 if enable else 0)


def soar_kernel_timing_read(kernel_id: int):
    ms, n = C.c_double(0.0), C.c_int64(0)
    rc = lib().soar_kernel_timing_read(kernel_id, C.byref(ms), C.byref(n))
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_kernel_timing_read")
    return ms.value, n.value


def soar_search_stats_enable(enable: bool) -> None:
    rc = lib().soar_search_stats_enable(1 if enable else 0)
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_search_stats_enable")


def soar_search_stats_read() -> dict:
    """Counters of the certified search since they were enabled: blocks, blocks handed over to the exhaustive
    loop, wave steps, wave steps with at least one block handed over."""
    c = (C.c_int64 * 4)()
    rc = lib().soar_search_stats_read(c)
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_search_stats_read")
    return {"blocks": c[0], "blocks_handed_over": c[1], "wave_steps": c[2], "wave_steps_with_hand_over": c[3]}


def soar_debug_arrival_plan(n_workgroups: int, workgroup: int):
    """(counters in use, this workgroup's counter, workgroups sharing it) of the kernels' arrival counting"""
    out = (C.c_uint32 * 3)(0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF)
    lib().soar_debug_arrival_plan(n_workgroups, workgroup, out)
    return out[0], out[1], out[2]


def soar_version() -> int:
    return int(lib().soar_version())


# ------------------------------------------------------------------ tensor-level helpers
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SOAR_BF16
    if t.dtype == torch.float32:
        return SOAR_FP32
    raise TypeError("weights must be bfloat16 or float32")


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _check_matrix(w: torch.Tensor):
    if not w.is_cuda:
        raise RuntimeError("soar: weights must live on the GPU (no CPU path exists)")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("weights must be 2-D with contiguous rows")
    return w.shape[0], w.shape[1], w.stride(0)


@dataclass
class Quantized:
    codes: torch.Tensor          # uint8 [rows, cols/2]
    scales: torch.Tensor         # uint8 [rows, cols/16]
    global_scale: Optional[torch.Tensor]   # float32 [1]; None for MXFP4 (the format has none)
    sse: torch.Tensor            # float64 [1]
    status: torch.Tensor         # int32 [1]
    iters_run: Optional[torch.Tensor] = None   # int32 [1], iterated path
    sse_trace: Optional[torch.Tensor] = None   # float64 [iters + 1], iterated path; NaN where not written


def new_workspace(rows: int, cols: int, params: soar_params, device) -> torch.Tensor:
    n = soar_workspace_bytes(rows, cols, params)
    if n == 0:
        raise SoarError(2, "soar_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def new_batch_workspace(descs: Sequence[soar_tensor_desc], params: soar_params, device) -> torch.Tensor:
    n = soar_batch_workspace_bytes(descs, params)
    if n == 0:
        raise SoarError(2, "soar_batch_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def quantize(w: torch.Tensor, method: int = SOAR_METHOD_SOAR, dss_radius: int = 4,
             search_mode: int = SOAR_SEARCH_AUTO, workspace: Optional[torch.Tensor] = None,
             out: Optional[Quantized] = None, tiles_per_wg: int = 0) -> Quantized:
    rows, cols, ld = _check_matrix(w)
    p = soar_default_params(method, dss_radius, search_mode, tiles_per_wg)
    dev = w.device
    if out is None:
        out = Quantized(torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev),
                        torch.empty((rows, cols // 16), dtype=torch.uint8, device=dev),
                        torch.empty(1, dtype=torch.float32, device=dev),
                        torch.empty(1, dtype=torch.float64, device=dev),
                        torch.empty(1, dtype=torch.int32, device=dev))
    if workspace is None:
        workspace = new_workspace(rows, cols, p, dev)
    rc = soar_quantize(w.data_ptr(), _dtype_code(w), rows, cols, ld, p, out.codes.data_ptr(),
                       out.scales.data_ptr(), out.global_scale.data_ptr(), out.sse.data_ptr(),
                       out.status.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_quantize")
    return out


def new_outputs(rows: int, cols: int, device, iters: int = 0) -> Quantized:
    """Output buffers for one tensor; iters > 0 adds the iterated path's two extra outputs."""
    q = Quantized(torch.empty((rows, cols // 2), dtype=torch.uint8, device=device),
                  torch.empty((rows, cols // 16), dtype=torch.uint8, device=device),
                  torch.empty(1, dtype=torch.float32, device=device),
                  torch.empty(1, dtype=torch.float64, device=device),
                  torch.empty(1, dtype=torch.int32, device=device))
    if iters > 0:
        q.iters_run = torch.zeros(1, dtype=torch.int32, device=device)
        q.sse_trace = torch.full((iters + 1,), float("nan"), dtype=torch.float64, device=device)
    return q


def make_desc(w: torch.Tensor, out: Quantized, amax_in: Optional[torch.Tensor] = None) -> soar_tensor_desc:
    """amax_in: float32 [1] on the GPU, the supplied tensor maximum (plain NVFP4 only)."""
    rows, cols, ld = _check_matrix(w)
    return soar_tensor_desc(w.data_ptr(), _dtype_code(w), rows, cols, ld, out.codes.data_ptr(),
                            out.scales.data_ptr(), out.global_scale.data_ptr(), out.sse.data_ptr(),
                            out.status.data_ptr(),
                            out.iters_run.data_ptr() if out.iters_run is not None else None,
                            out.sse_trace.data_ptr() if out.sse_trace is not None else None,
                            amax_in.data_ptr() if amax_in is not None else None)


def quantize_iter(w: torch.Tensor, params: soar_params, workspace: Optional[torch.Tensor] = None,
                  out: Optional[Quantized] = None) -> Quantized:
    """One tensor through the iterated path (soar_quantize_batch with n = 1), with the error trace."""
    rows, cols, _ = _check_matrix(w)
    if out is None:
        out = new_outputs(rows, cols, w.device, params.iters)
    desc = make_desc(w, out)
    if workspace is None:
        workspace = new_batch_workspace([desc], params, w.device)
    quantize_batch([desc], params, workspace)
    return out


def quantize_batch(descs: Sequence[soar_tensor_desc], params: soar_params, workspace: torch.Tensor) -> None:
    rc = soar_quantize_batch(descs, params, workspace.data_ptr(), workspace.numel(), _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_quantize_batch")


def quantize_rtn_amax(w: torch.Tensor, amax_in: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                      out: Optional[Quantized] = None) -> Quantized:
    """Plain NVFP4 (Sec. 3.1) of one tensor with its maximum supplied: a single pass over the data."""
    rows, cols, _ = _check_matrix(w)
    if amax_in.dtype != torch.float32 or not amax_in.is_cuda:
        raise TypeError("amax_in must be a float32 tensor on the GPU")
    if out is None:
        out = new_outputs(rows, cols, w.device)
    p = soar_default_params(SOAR_METHOD_RTN, 0)
    desc = make_desc(w, out, amax_in)
    if workspace is None:
        workspace = new_batch_workspace([desc], p, w.device)
    quantize_batch([desc], p, workspace)
    return out


def quantize_tensors(weights: Sequence[torch.Tensor], params: Optional[soar_params] = None,
                     workspace: Optional[torch.Tensor] = None) -> list:
    """The linear layers of a model in one soar_quantize_batch call: allocates the outputs (with the
    trace buffers when the parameters select the iterated path), one shared workspace, and enqueues
    everything on the current stream.  Returns one Quantized per tensor, in order."""
    if not weights:
        return []
    if params is None:
        params = soar_default_params()
    iterated = (params.iters != 1 or params.n_beta != 1 or params.beta_lo != 1.0 or
                params.dd_mode != SOAR_DD_WINDOW or params.method in (SOAR_METHOD_CJSO_ONLY, SOAR_METHOD_DSS_ONLY))
    outs = []
    for w in weights:
        rows, cols, _ = _check_matrix(w)
        outs.append(new_outputs(rows, cols, w.device, params.iters if iterated else 0))
    descs = [make_desc(w, o) for w, o in zip(weights, outs)]
    if workspace is None:
        workspace = new_batch_workspace(descs, params, weights[0].device)
    quantize_batch(descs, params, workspace)
    return outs


def dequantize(q: Quantized, out_dtype=torch.bfloat16) -> torch.Tensor:
    rows, cols = q.scales.shape[0], q.scales.shape[1] * 16
    out = torch.empty((rows, cols), dtype=out_dtype, device=q.codes.device)
    rc = soar_dequantize(q.codes.data_ptr(), q.scales.data_ptr(), q.global_scale.data_ptr(), rows, cols,
                         _dtype_code(out), out.data_ptr(), cols, _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_dequantize")
    return out


def recon_error(w: torch.Tensor, q: Quantized) -> torch.Tensor:
    rows, cols, ld = _check_matrix(w)
    sse = torch.empty(1, dtype=torch.float64, device=w.device)
    rc = soar_recon_error(w.data_ptr(), _dtype_code(w), rows, cols, ld, q.codes.data_ptr(),
                          q.scales.data_ptr(), q.global_scale.data_ptr(), sse.data_ptr(), _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_recon_error")
    return sse


def stored_desc(q: Quantized, w: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                sse: Optional[torch.Tensor] = None) -> "soar_stored_desc":
    """Descriptor of one stored tensor: `w` and `sse` for Eq. 4, `out` for Eq. 3 (the tensors must stay alive
    until the call that uses the descriptor has been enqueued)."""
    m = w if w is not None else out
    rows, cols, ld = _check_matrix(m)
    d = soar_stored_desc()
    d.d_codes, d.d_scales, d.d_global_scale = q.codes.data_ptr(), q.scales.data_ptr(), q.global_scale.data_ptr()
    d.rows, d.cols, d.ld_elems, d.dtype = rows, cols, ld, _dtype_code(m)
    d.d_w = w.data_ptr() if w is not None else None
    d.d_out = out.data_ptr() if out is not None else None
    d.d_sse = sse.data_ptr() if sse is not None else None
    return d


def dequantize_batch(qs: Sequence[Quantized], out_dtype=torch.bfloat16) -> list:
    """Eq. 3 for a list of stored tensors in a handful of launches."""
    outs = [torch.empty((q.scales.shape[0], q.scales.shape[1] * 16), dtype=out_dtype, device=q.codes.device) for q in qs]
    rc = soar_dequantize_batch([stored_desc(q, out=o) for q, o in zip(qs, outs)], _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_dequantize_batch")
    return outs


def recon_error_batch(weights: Sequence[torch.Tensor], qs: Sequence[Quantized]) -> torch.Tensor:
    """Eq. 4 for a list of tensors in a handful of launches: one binary64 sum per tensor."""
    if not weights:
        return torch.empty(0, dtype=torch.float64)
    sses = torch.empty(len(weights), dtype=torch.float64, device=weights[0].device)
    rc = soar_recon_error_batch([stored_desc(q, w=w, sse=sses[k:k + 1]) for k, (w, q) in enumerate(zip(weights, qs))],
                                _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_recon_error_batch")
    return sses


# ------------------------------------------------------------------ MXFP4
def mx_new_outputs(rows: int, cols: int, device) -> Quantized:
    return Quantized(torch.empty((rows, cols // 2), dtype=torch.uint8, device=device),
                     torch.empty((rows, cols // 32), dtype=torch.uint8, device=device),
                     None,
                     torch.empty(1, dtype=torch.float64, device=device),
                     torch.empty(1, dtype=torch.int32, device=device))


def mx_quantize(w: torch.Tensor, params: soar_mx_params, workspace: Optional[torch.Tensor] = None,
                out: Optional[Quantized] = None) -> Quantized:
    """MXFP4 conversion of one tensor (plain or with the decoupled scale search); scales are E8M0 bytes."""
    rows, cols, ld = _check_matrix(w)
    if out is None:
        out = mx_new_outputs(rows, cols, w.device)
    if workspace is None:
        n = soar_mxfp4_workspace_bytes(rows, cols, params)
        if n == 0:
            raise SoarError(2, "soar_mxfp4_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=w.device)
    rc = soar_mxfp4_quantize(w.data_ptr(), _dtype_code(w), rows, cols, ld, params, out.codes.data_ptr(),
                             out.scales.data_ptr(), out.sse.data_ptr(), out.status.data_ptr(),
                             workspace.data_ptr(), workspace.numel(), _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_mxfp4_quantize")
    return out


def mx_make_desc(w: torch.Tensor, out: Quantized) -> soar_mx_tensor_desc:
    rows, cols, ld = _check_matrix(w)
    return soar_mx_tensor_desc(w.data_ptr(), _dtype_code(w), rows, cols, ld, out.codes.data_ptr(),
                               out.scales.data_ptr(), out.sse.data_ptr(), out.status.data_ptr())


def mx_quantize_batch(descs: Sequence[soar_mx_tensor_desc], params: soar_mx_params,
                      workspace: Optional[torch.Tensor] = None, device=None) -> None:
    if workspace is None:
        n = soar_mxfp4_batch_workspace_bytes(descs, params)
        if n == 0:
            raise SoarError(2, "soar_mxfp4_batch_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=device or "cuda")
    rc = soar_mxfp4_quantize_batch(descs, params, workspace.data_ptr(), workspace.numel(), _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_mxfp4_quantize_batch")


def mx_stored_desc(q: Quantized, out: torch.Tensor) -> "soar_stored_desc":
    rows, cols, ld = _check_matrix(out)
    d = soar_stored_desc()
    d.d_codes, d.d_scales = q.codes.data_ptr(), q.scales.data_ptr()
    d.rows, d.cols, d.ld_elems, d.dtype = rows, cols, ld, _dtype_code(out)
    d.d_out = out.data_ptr()
    return d


def mx_dequantize_batch(qs: Sequence[Quantized], out_dtype=torch.bfloat16) -> list:
    """MXFP4 tensors back to bf16 / fp32 in a handful of launches."""
    outs = [torch.empty((q.scales.shape[0], q.scales.shape[1] * 32), dtype=out_dtype, device=q.codes.device) for q in qs]
    rc = soar_mxfp4_dequantize_batch([mx_stored_desc(q, o) for q, o in zip(qs, outs)], _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_mxfp4_dequantize_batch")
    return outs


def mx_dequantize(q: Quantized, out_dtype=torch.bfloat16) -> torch.Tensor:
    rows, cols = q.scales.shape[0], q.scales.shape[1] * 32
    out = torch.empty((rows, cols), dtype=out_dtype, device=q.codes.device)
    rc = soar_mxfp4_dequantize(q.codes.data_ptr(), q.scales.data_ptr(), rows, cols, _dtype_code(out),
                               out.data_ptr(), cols, _stream())
    if rc != SOAR_OK:
        raise SoarError(rc, "soar_mxfp4_dequantize")
    return out
