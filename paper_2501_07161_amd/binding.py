"""ctypes binding of libqv2.so: same names as the C ABI, argument marshalling only.

Every step of the sensitivity pass runs inside the native library; PyTorch is
used for device memory and streams.  There is no fallback: if the library has
not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# QV2_LIB_PATH selects another build of the same library (tuning variants).
LIB_PATH = os.environ.get("QV2_LIB_PATH") or os.path.join(_HERE, "libqv2.so")

QV2_OK = 0
QV2_ERR_NULL, QV2_ERR_SHAPE, QV2_ERR_SCHEME, QV2_ERR_WORKSPACE = -1, -2, -3, -4
QV2_ERR_NONFINITE, QV2_ERR_HIP, QV2_ERR_ALIGN, QV2_ERR_IO, QV2_ERR_NOMEM, QV2_ERR_STATE = -5, -6, -7, -8, -9, -10
QV2_STATIC_SCRATCH_BYTES = 64 << 20
QV2_ASYM_TENSOR, QV2_SYM_TENSOR, QV2_SYM_CHANNEL = 0, 1, 2

EXPORTS = (
    "qv2_plan_create", "qv2_plan_destroy", "qv2_plan_num_tensors", "qv2_plan_num_segments",
    "qv2_plan_segment_begin", "qv2_plan_num_tiles", "qv2_plan_num_quant_tiles",
    "qv2_plan_num_pair_tiles", "qv2_plan_num_single_read_elements", "qv2_plan_upload", "qv2_plan_device_bytes",
    "qv2_calibrate_fakequant_pair_metrics_noalloc",
    "qv2_workspace_bytes", "qv2_calibrate", "qv2_fakequant_metrics", "qv2_pair_metrics",
    "qv2_fakequant_pair_metrics", "qv2_calibrate_fakequant_pair_metrics", "qv2_calibrate_fakequant_pair_metrics_cos",
    "qv2_fakequant_pair_metrics_cos", "qv2_cosine_finalize",
    "qv2_plan_set_timing", "qv2_plan_time_only", "qv2_sensitivity_pass_begin", "qv2_sensitivity_pass_end",
    "qv2_plan_kernel_ms", "qv2_plan_kernels_ms", "qv2_histogram_workspace_bytes", "qv2_histogram",
    "qv2_kl_divergence", "qv2_bn_fold", "qv2_regroup_for_fusion", "qv2_tensor_sums_fold",
    "qv2_finalize_tensors",
    "qv2_finalize", "qv2_pair_finalize", "qv2_rank_config_default", "qv2_rank", "qv2_rank_tensors", "qv2_sensitivity_pass", "qv2_write_config",
    "qv2_baseline_order", "qv2_bops_reduction_pct", "qv2_bops_select",
    "qv2_status_string",
)


class qv2_tensor(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("qrun", ctypes.c_void_p), ("codes", ctypes.c_void_p),
                ("numel", ctypes.c_int64), ("channels", ctypes.c_int32), ("scheme", ctypes.c_int32),
                ("kind", ctypes.c_int32), ("layer", ctypes.c_int32)]


class qv2_rank_config(ctypes.Structure):
    _fields_ = [("alpha_w", ctypes.c_double), ("alpha_a", ctypes.c_double),
                ("mse_factor", ctypes.c_double), ("sqnr_cap_db", ctypes.c_double),
                ("mse_source", ctypes.c_int32), ("_pad", ctypes.c_int32)]


# numpy views of the POD records the library reads and writes
QPARAMS = np.dtype([("min", "<f4"), ("max", "<f4"), ("scale", "<f4"), ("inv_scale", "<f4"),
                    ("zp", "<i4"), ("_pad", "<i4")])
SUMS = np.dtype([("sum_x", "<f8"), ("sum_x2", "<f8"), ("sum_e2", "<f8"), ("n", "<i8")])
PAIR_SUMS = np.dtype([("sum_ref2", "<f8"), ("sum_d2", "<f8"), ("n", "<i8"), ("_pad", "<i8")])
METRICS = np.dtype([("mse", "<f8"), ("sqnr_db", "<f8"), ("mean", "<f8"), ("var", "<f8"),
                    ("absmax", "<f4"), ("min", "<f4"), ("max", "<f4"), ("_pad", "<i4")])
TENSOR_SUMS = np.dtype([("sum_x", "<f8"), ("sum_x2", "<f8"), ("sum_e2", "<f8"), ("n", "<i8"),
                        ("min", "<f4"), ("max", "<f4"), ("_pad", "<i4", (2,))])
assert TENSOR_SUMS.itemsize == 48
assert QPARAMS.itemsize == 24 and SUMS.itemsize == 32 and PAIR_SUMS.itemsize == 32
assert METRICS.itemsize == 48

_lib = None


class QV2Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().qv2_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} ({status})")


def lib():
    """Load libqv2.so (built by paper_2501_07161_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2501_07161_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.qv2_plan_create.argtypes = [ctypes.POINTER(qv2_tensor), i32, ctypes.POINTER(vp)]
        L.qv2_plan_destroy.argtypes = [vp]
        L.qv2_plan_destroy.restype = None
        L.qv2_plan_num_tensors.argtypes = [vp]
        L.qv2_plan_num_tensors.restype = i32
        for n in ("qv2_plan_num_segments", "qv2_plan_num_tiles", "qv2_plan_num_quant_tiles",
                  "qv2_plan_num_pair_tiles", "qv2_plan_num_single_read_elements"):
            getattr(L, n).argtypes = [vp]
            getattr(L, n).restype = i64
        L.qv2_plan_segment_begin.argtypes = [vp, i32]
        L.qv2_plan_segment_begin.restype = i64
        L.qv2_workspace_bytes.argtypes = [vp]
        L.qv2_workspace_bytes.restype = sz
        L.qv2_plan_upload.argtypes = [vp, vp]
        L.qv2_plan_device_bytes.argtypes = [vp]
        L.qv2_plan_device_bytes.restype = sz
        L.qv2_calibrate_fakequant_pair_metrics_noalloc.argtypes = [vp, vp, vp, vp, vp]
        L.qv2_calibrate.argtypes = [vp, vp, vp, vp, sz, vp]
        L.qv2_fakequant_metrics.argtypes = [vp, vp, vp, vp, sz, vp]
        L.qv2_pair_metrics.argtypes = [vp, vp, vp, sz, vp]
        L.qv2_fakequant_pair_metrics.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.qv2_calibrate_fakequant_pair_metrics.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.qv2_fakequant_pair_metrics_cos.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qv2_calibrate_fakequant_pair_metrics_cos.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.qv2_cosine_finalize.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.qv2_histogram_workspace_bytes.argtypes = [vp, i32]
        L.qv2_histogram_workspace_bytes.restype = sz
        L.qv2_histogram.argtypes = [vp, vp, i32, vp, vp, vp, sz, vp]
        L.qv2_kl_divergence.argtypes = [vp, vp, i32, ctypes.c_double, vp]
        L.qv2_bn_fold.argtypes = [vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        L.qv2_regroup_for_fusion.argtypes = [vp, vp, i32, vp]
        L.qv2_tensor_sums_fold.argtypes = [vp, vp, vp, vp, vp]
        L.qv2_finalize_tensors.argtypes = [vp, i32, vp]
        L.qv2_plan_set_timing.argtypes = [vp, i32]
        L.qv2_plan_time_only.argtypes = [vp, i32]
        L.qv2_sensitivity_pass_begin.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp, i32]
        L.qv2_sensitivity_pass_end.argtypes = [vp, vp, i32, vp, i32, ctypes.POINTER(qv2_rank_config),
                                               vp, vp, vp, vp, vp]
        L.qv2_plan_kernel_ms.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_float)]
        L.qv2_plan_kernels_ms.argtypes = [vp, vp]
        L.qv2_finalize.argtypes = [vp, vp, vp, vp]
        L.qv2_pair_finalize.argtypes = [vp, i32, vp, vp]
        L.qv2_rank_config_default.argtypes = [ctypes.POINTER(qv2_rank_config)]
        L.qv2_rank_config_default.restype = None
        L.qv2_rank.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.POINTER(qv2_rank_config), vp, vp]
        L.qv2_rank_tensors.argtypes = [vp, vp, vp, vp, i32, ctypes.POINTER(qv2_rank_config), vp, vp]
        L.qv2_sensitivity_pass.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp, vp, i32, ctypes.POINTER(qv2_rank_config),
                                           vp, vp, vp, vp, vp]
        L.qv2_write_config.argtypes = [ctypes.c_char_p, vp, vp, i32]
        L.qv2_baseline_order.argtypes = [i32, vp, i32, vp]
        L.qv2_bops_reduction_pct.argtypes = [vp, vp, i32, vp]
        L.qv2_bops_select.argtypes = [vp, vp, i32, ctypes.c_double, vp, vp, vp]
        L.qv2_status_string.argtypes = [ctypes.c_int]
        L.qv2_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(st: int, where: str):
    if st != QV2_OK:
        raise QV2Error(st, where)


def _ptr(buf) -> Optional[int]:
    """Address of a torch tensor / numpy array / int / None."""
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if isinstance(buf, np.ndarray):
        return buf.ctypes.data
    return buf.data_ptr()


def _dev(buf, need_bytes: int, what: str, elem_size: Optional[int] = None, optional: bool = False,
         dtype: Optional[str] = None):
    """Address of a device buffer after checking what can be checked on the host: a torch
    tensor must live on the GPU, be contiguous and hold at least `need_bytes` (and have
    `elem_size`-byte elements when given).  A kernel handed a short or host buffer would fault
    the GPU, so these are refused here.  Raw integer addresses are passed through unchecked."""
    if buf is None:
        if optional:
            return None
        raise QV2Error(QV2_ERR_NULL, what)
    if isinstance(buf, int):
        return buf
    if not getattr(buf, "is_cuda", False):
        raise QV2Error(QV2_ERR_NULL, f"{what}: not a device tensor")
    if not buf.is_contiguous():
        raise QV2Error(QV2_ERR_SHAPE, f"{what}: not contiguous")
    if elem_size is not None and buf.element_size() != elem_size:
        raise QV2Error(QV2_ERR_SHAPE, f"{what}: {buf.element_size()}-byte elements, {elem_size} expected")
    if dtype is not None and str(getattr(buf, "dtype", dtype)) != dtype:
        raise QV2Error(QV2_ERR_SHAPE, f"{what}: dtype {buf.dtype}, {dtype} expected")
    have = buf.numel() * buf.element_size()
    if have < need_bytes:
        raise QV2Error(QV2_ERR_SHAPE, f"{what}: holds {have} bytes, {need_bytes} needed")
    return buf.data_ptr()


def _ws(plan, d_workspace, workspace_bytes, where: str):
    """(address, byte count) of a workspace argument."""
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size()
    return _dev(d_workspace, 0 if isinstance(d_workspace, int) else workspace_bytes, f"{where}: workspace"), \
        workspace_bytes


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


@dataclass
class TensorArg:
    """One row of the layer table.  x / qrun / codes are torch device tensors
    (or raw device addresses); the plan keeps references to them."""
    x: object
    numel: int
    scheme: int = QV2_ASYM_TENSOR
    channels: int = 1
    qrun: object = None
    codes: object = None
    kind: int = 0
    layer: int = 0


class Plan:
    """Owner of a native qv2_plan handle."""

    def __init__(self, handle: int, rows: Sequence[TensorArg]):
        self.handle = handle
        self.rows = list(rows)            # keeps the device tensors alive
        L = lib()
        self.num_tensors = L.qv2_plan_num_tensors(handle)
        self.num_segments = L.qv2_plan_num_segments(handle)
        self.num_tiles = L.qv2_plan_num_tiles(handle)
        self.num_quant_tiles = L.qv2_plan_num_quant_tiles(handle)
        self.num_pair_tiles = L.qv2_plan_num_pair_tiles(handle)
        self.num_single_read_elements = L.qv2_plan_num_single_read_elements(handle)
        self.workspace_bytes = L.qv2_workspace_bytes(handle)
        self.segment_begin = [L.qv2_plan_segment_begin(handle, t) for t in range(self.num_tensors)]

    def close(self):
        if self.handle:
            lib().qv2_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def qv2_plan_create(rows: Sequence[TensorArg]) -> Plan:
    n = len(rows)
    arr = (qv2_tensor * max(n, 1))()
    for i, r in enumerate(rows):
        nel = int(r.numel)
        arr[i] = qv2_tensor(_dev(r.x, 4 * nel, f"qv2_plan_create: x of tensor {i}", 4, dtype="torch.float32"),
                            _dev(r.qrun, 4 * nel, f"qv2_plan_create: qrun of tensor {i}", 4, optional=True,
                                 dtype="torch.float32"),
                            _dev(r.codes, nel, f"qv2_plan_create: codes of tensor {i}", 1, optional=True),
                            nel, int(r.channels), int(r.scheme), int(r.kind), int(r.layer))
    h = ctypes.c_void_p()
    _check(lib().qv2_plan_create(arr, n, ctypes.byref(h)), "qv2_plan_create")
    return Plan(h.value, rows)


KERNEL_IDS = {"k_stats_stream": 0, "k_stats_rows": 1, "k_quant_stream": 2, "k_quant_rows": 3,
              "k_pair_stream": 4, "k_quantpair_stream": 5, "k_quantpair_rows": 6, "k_hist": 7,
              "k_single_read_rows": 8, "k_statspair_stream": 9}


def qv2_plan_set_timing(plan: Plan, enable: bool):
    _check(lib().qv2_plan_set_timing(plan.handle, int(bool(enable))), "qv2_plan_set_timing")


def qv2_plan_time_only(plan: Plan, kernel):
    """Bracket only this tile kernel (name or id) with events; None = all of them again."""
    kid = -1 if kernel is None else KERNEL_IDS[kernel] if isinstance(kernel, str) else int(kernel)
    _check(lib().qv2_plan_time_only(plan.handle, kid), "qv2_plan_time_only")


def qv2_plan_kernel_ms(plan: Plan, kernel) -> float:
    """Duration of the last launch of a tile kernel (name or id); the stream must be synchronised."""
    ms = ctypes.c_float()
    kid = KERNEL_IDS[kernel] if isinstance(kernel, str) else int(kernel)
    _check(lib().qv2_plan_kernel_ms(plan.handle, kid, ctypes.byref(ms)), "qv2_plan_kernel_ms")
    return ms.value


def qv2_plan_kernels_ms(plan: Plan, out=None):
    """Durations of the most recent launch of every tile kernel, indexed by KERNEL_IDS
    (float32 array of len(KERNEL_IDS); `out` is reused when given)."""
    import numpy as np
    if out is None:
        out = np.zeros(len(KERNEL_IDS), dtype=np.float32)
    _check(lib().qv2_plan_kernels_ms(plan.handle, out.ctypes.data), "qv2_plan_kernels_ms")
    return out


def qv2_plan_upload(plan: Plan, stream=None):
    """Puts the plan's tables on the current device now (device calls do it on first use otherwise)."""
    _check(lib().qv2_plan_upload(plan.handle, _stream(stream)), "qv2_plan_upload")


def qv2_plan_device_bytes(plan: Plan) -> int:
    return lib().qv2_plan_device_bytes(plan.handle)


def qv2_workspace_bytes(plan: Plan) -> int:
    return lib().qv2_workspace_bytes(plan.handle)


def _seg_args(plan: Plan, d_params, d_sums, where: str):
    return (_dev(d_params, plan.num_segments * QPARAMS.itemsize, f"{where}: d_params"),
            _dev(d_sums, plan.num_segments * SUMS.itemsize, f"{where}: d_sums"))


def _pair_arg(plan: Plan, d_pair_sums, where: str, optional: bool = False):
    return _dev(d_pair_sums, plan.num_tensors * PAIR_SUMS.itemsize, f"{where}: d_pair_sums", optional=optional)


def _cos_args(plan: Plan, d_seg_xxhat, d_pair_xq, where: str):
    return (_dev(d_seg_xxhat, plan.num_segments * 8, f"{where}: d_seg_xxhat"),
            _dev(d_pair_xq, plan.num_tensors * 8, f"{where}: d_pair_xq"))


def qv2_calibrate(plan: Plan, d_params, d_sums, d_workspace, workspace_bytes=None, stream=None):
    w = "qv2_calibrate"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_calibrate(plan.handle, *_seg_args(plan, d_params, d_sums, w), ws, wb, _stream(stream)), w)


def qv2_fakequant_metrics(plan: Plan, d_params, d_sums, d_workspace, workspace_bytes=None, stream=None):
    w = "qv2_fakequant_metrics"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_fakequant_metrics(plan.handle, *_seg_args(plan, d_params, d_sums, w), ws, wb,
                                       _stream(stream)), w)


def qv2_pair_metrics(plan: Plan, d_pair_sums, d_workspace, workspace_bytes=None, stream=None):
    w = "qv2_pair_metrics"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_pair_metrics(plan.handle, _pair_arg(plan, d_pair_sums, w), ws, wb, _stream(stream)), w)


def qv2_fakequant_pair_metrics(plan: Plan, d_params, d_sums, d_pair_sums, d_workspace,
                               workspace_bytes=None, stream=None):
    w = "qv2_fakequant_pair_metrics"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_fakequant_pair_metrics(plan.handle, *_seg_args(plan, d_params, d_sums, w),
                                            _pair_arg(plan, d_pair_sums, w), ws, wb, _stream(stream)), w)


def qv2_calibrate_fakequant_pair_metrics(plan: Plan, d_params, d_sums, d_pair_sums, d_workspace,
                                         workspace_bytes=None, stream=None):
    """d_pair_sums may be None (no comparison with qrun)."""
    w = "qv2_calibrate_fakequant_pair_metrics"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_calibrate_fakequant_pair_metrics(
        plan.handle, *_seg_args(plan, d_params, d_sums, w), _pair_arg(plan, d_pair_sums, w, optional=True),
        ws, wb, _stream(stream)), w)


def qv2_calibrate_fakequant_pair_metrics_noalloc(plan: Plan, d_params, d_sums, d_pair_sums, stream=None):
    """The single call on the library's own fixed device array: no workspace, no allocation.
    The plan must have been uploaded (qv2_plan_upload or an earlier device call)."""
    w = "qv2_calibrate_fakequant_pair_metrics_noalloc"
    _check(lib().qv2_calibrate_fakequant_pair_metrics_noalloc(
        plan.handle, *_seg_args(plan, d_params, d_sums, w), _pair_arg(plan, d_pair_sums, w, optional=True),
        _stream(stream)), w)


def qv2_calibrate_fakequant_pair_metrics_cos(plan: Plan, d_params, d_sums, d_pair_sums, d_seg_xxhat, d_pair_xq,
                                             d_workspace, workspace_bytes=None, stream=None):
    w = "qv2_calibrate_fakequant_pair_metrics_cos"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_calibrate_fakequant_pair_metrics_cos(
        plan.handle, *_seg_args(plan, d_params, d_sums, w), _pair_arg(plan, d_pair_sums, w),
        *_cos_args(plan, d_seg_xxhat, d_pair_xq, w), ws, wb, _stream(stream)), w)


def qv2_fakequant_pair_metrics_cos(plan: Plan, d_params, d_sums, d_pair_sums, d_seg_xxhat, d_pair_xq,
                                   d_workspace, workspace_bytes=None, stream=None):
    w = "qv2_fakequant_pair_metrics_cos"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    _check(lib().qv2_fakequant_pair_metrics_cos(
        plan.handle, *_seg_args(plan, d_params, d_sums, w), _pair_arg(plan, d_pair_sums, w),
        *_cos_args(plan, d_seg_xxhat, d_pair_xq, w), ws, wb, _stream(stream)), w)


def qv2_cosine_finalize(plan: Plan, h_sums, h_seg_xxhat, h_pair, h_pair_xq, strict: bool = True):
    """Returns (cos(x, xhat), cos(x, qrun)) per tensor."""
    hs = np.ascontiguousarray(h_sums, dtype=SUMS)
    hp = np.ascontiguousarray(h_pair, dtype=PAIR_SUMS)
    sx = _f64(h_seg_xxhat)
    px = _f64(h_pair_xq)
    if hs.size != plan.num_segments or sx.size != plan.num_segments or hp.size != plan.num_tensors \
            or px.size != plan.num_tensors:
        raise QV2Error(QV2_ERR_SHAPE, "qv2_cosine_finalize")
    cq = np.zeros(plan.num_tensors, np.float64)
    cp = np.zeros(plan.num_tensors, np.float64)
    st = lib().qv2_cosine_finalize(plan.handle, hs.ctypes.data, sx.ctypes.data, hp.ctypes.data,
                                   px.ctypes.data, cq.ctypes.data, cp.ctypes.data)
    if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
        raise QV2Error(st, "qv2_cosine_finalize")
    return cq, cp


def qv2_histogram_workspace_bytes(plan: Plan, nbins: int) -> int:
    return lib().qv2_histogram_workspace_bytes(plan.handle, int(nbins))


def qv2_histogram(plan: Plan, d_params, nbins: int, d_hist_x, d_hist_q, d_workspace, workspace_bytes=None,
                  stream=None):
    w = "qv2_histogram"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    hb = plan.num_tensors * max(int(nbins), 0) * 8
    _check(lib().qv2_histogram(plan.handle,
                               _dev(d_params, plan.num_segments * QPARAMS.itemsize, f"{w}: d_params"), int(nbins),
                               _dev(d_hist_x, hb, f"{w}: d_hist_x", 8),
                               _dev(d_hist_q, hb, f"{w}: d_hist_q", 8, optional=True), ws, wb, _stream(stream)), w)


def qv2_kl_divergence(hist_p, hist_q, eps: float = 0.0) -> float:
    hp = np.ascontiguousarray(hist_p, dtype=np.uint64)
    hq = np.ascontiguousarray(hist_q, dtype=np.uint64)
    if hp.size != hq.size:
        raise QV2Error(QV2_ERR_SHAPE, "qv2_kl_divergence")
    out = ctypes.c_double()
    _check(lib().qv2_kl_divergence(hp.ctypes.data, hq.ctypes.data, hp.size, float(eps), ctypes.addressof(out)),
           "qv2_kl_divergence")
    return out.value


def qv2_bn_fold(d_w, channels: int, inner: int, d_gamma, d_var, d_w_out, d_bias=None, d_mean=None,
                d_beta=None, d_bias_out=None, stream=None):
    w, c, n = "qv2_bn_fold", max(int(channels), 0), max(int(channels), 0) * max(int(inner), 0)
    _check(lib().qv2_bn_fold(_dev(d_w, 4 * n, f"{w}: d_w", 4), int(channels), int(inner),
                             _dev(d_gamma, 4 * c, f"{w}: d_gamma", 4), _dev(d_var, 4 * c, f"{w}: d_var", 4),
                             _dev(d_bias, 4 * c, f"{w}: d_bias", 4, optional=True),
                             _dev(d_mean, 4 * c, f"{w}: d_mean", 4, optional=True),
                             _dev(d_beta, 4 * c, f"{w}: d_beta", 4, optional=True),
                             _dev(d_w_out, 4 * n, f"{w}: d_w_out", 4),
                             _dev(d_bias_out, 4 * c, f"{w}: d_bias_out", 4, optional=True), _stream(stream)), w)


def qv2_write_config(path: str, keep_fp32, layer_names=None):
    """Writes the per-layer bit-width table (32 for kept-in-fp32 layers, 8 otherwise)."""
    keep = np.ascontiguousarray(keep_fp32, dtype=np.uint8)
    n = len(keep)
    names = None
    if layer_names is not None:
        if len(layer_names) != n:
            raise QV2Error(QV2_ERR_SHAPE, "qv2_write_config")
        names = (ctypes.c_char_p * n)(*[s.encode() for s in layer_names])
    _check(lib().qv2_write_config(os.fsencode(path), keep.ctypes.data, names, n), "qv2_write_config")


def qv2_regroup_for_fusion(order, group_id) -> np.ndarray:
    o = np.ascontiguousarray(order, dtype=np.int32)
    g = np.ascontiguousarray(group_id, dtype=np.int32)
    if len(o) != len(g):
        raise QV2Error(QV2_ERR_SHAPE, "qv2_regroup_for_fusion")
    out = np.zeros(max(len(o), 1), np.int32)
    _check(lib().qv2_regroup_for_fusion(o.ctypes.data, g.ctypes.data, len(o), out.ctypes.data),
           "qv2_regroup_for_fusion")
    return out[:len(o)]


def qv2_tensor_sums_fold(plan: Plan, d_params, d_sums, d_tensor_sums, stream=None):
    w = "qv2_tensor_sums_fold"
    _check(lib().qv2_tensor_sums_fold(plan.handle, *_seg_args(plan, d_params, d_sums, w),
                                      _dev(d_tensor_sums, plan.num_tensors * TENSOR_SUMS.itemsize,
                                           f"{w}: d_tensor_sums"), _stream(stream)), w)


def qv2_finalize_tensors(h_tensor_sums: np.ndarray, strict: bool = True) -> np.ndarray:
    ht = np.ascontiguousarray(h_tensor_sums, dtype=TENSOR_SUMS)
    out = np.zeros(ht.size, dtype=METRICS)
    st = lib().qv2_finalize_tensors(ht.ctypes.data, ht.size, out.ctypes.data)
    if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
        raise QV2Error(st, "qv2_finalize_tensors")
    return out


def qv2_finalize(plan: Plan, h_params: np.ndarray, h_sums: np.ndarray, strict: bool = True) -> np.ndarray:
    """Host fp64 metrics per tensor from host copies of params and sums."""
    hp = np.ascontiguousarray(h_params, dtype=QPARAMS)
    hs = np.ascontiguousarray(h_sums, dtype=SUMS)
    if hp.size != plan.num_segments or hs.size != plan.num_segments:
        raise QV2Error(QV2_ERR_SHAPE, "qv2_finalize")
    out = np.zeros(plan.num_tensors, dtype=METRICS)
    st = lib().qv2_finalize(plan.handle, hp.ctypes.data, hs.ctypes.data, out.ctypes.data)
    if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
        raise QV2Error(st, "qv2_finalize")
    return out


def qv2_pair_finalize(h_pair: np.ndarray, strict: bool = True):
    hp = np.ascontiguousarray(h_pair, dtype=PAIR_SUMS)
    mse = np.zeros(hp.size, np.float64)
    sqnr = np.zeros(hp.size, np.float64)
    st = lib().qv2_pair_finalize(hp.ctypes.data, hp.size, mse.ctypes.data, sqnr.ctypes.data)
    if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
        raise QV2Error(st, "qv2_pair_finalize")
    return mse, sqnr


def qv2_rank_config_default() -> qv2_rank_config:
    c = qv2_rank_config()
    lib().qv2_rank_config_default(ctypes.byref(c))
    return c


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def qv2_rank(w_sqnr_db, a_sqnr_db, w_mse, a_mse, layer_pos=None, cfg: Optional[qv2_rank_config] = None,
             n_layers: Optional[int] = None):
    """Returns (order, score) as numpy arrays; order[0] = most sensitive layer."""
    ws, as_, wm, am = _f64(w_sqnr_db), _f64(a_sqnr_db), _f64(w_mse), _f64(a_mse)
    if n_layers is None:
        n_layers = next((len(a) for a in (ws, as_, wm, am) if a is not None), 0)
    for a in (ws, as_, wm, am):
        if a is not None and len(a) != n_layers:
            raise QV2Error(QV2_ERR_SHAPE, "qv2_rank")
    pos = None if layer_pos is None else np.ascontiguousarray(layer_pos, dtype=np.int32)
    if pos is not None and len(pos) != n_layers:
        raise QV2Error(QV2_ERR_SHAPE, "qv2_rank")
    order = np.zeros(max(n_layers, 1), np.int32)
    score = np.zeros(max(n_layers, 1), np.float64)
    _check(lib().qv2_rank(_ptr(ws), _ptr(as_), _ptr(wm), _ptr(am), _ptr(pos), n_layers,
                          ctypes.byref(cfg) if cfg is not None else None,
                          order.ctypes.data, score.ctypes.data), "qv2_rank")
    return order[:n_layers], score[:n_layers]


def qv2_rank_tensors(plan: "Plan", h_tensor_sums, h_pair_sums, n_layers: int, layer_pos=None,
                     cfg: Optional[qv2_rank_config] = None):
    """Ranking straight from the per-tensor records (TENSOR_SUMS / PAIR_SUMS arrays of
    plan.num_tensors entries).  Returns (order, score)."""
    ts = np.ascontiguousarray(h_tensor_sums)
    ps = None if h_pair_sums is None else np.ascontiguousarray(h_pair_sums)
    if len(ts) != plan.num_tensors or (ps is not None and len(ps) != plan.num_tensors):
        raise QV2Error(QV2_ERR_SHAPE, "qv2_rank_tensors")
    pos = None if layer_pos is None else np.ascontiguousarray(layer_pos, dtype=np.int32)
    if pos is not None and len(pos) != n_layers:
        raise QV2Error(QV2_ERR_SHAPE, "qv2_rank_tensors")
    order = np.zeros(max(n_layers, 1), np.int32)
    score = np.zeros(max(n_layers, 1), np.float64)
    _check(lib().qv2_rank_tensors(plan.handle, ts.ctypes.data, ps.ctypes.data if ps is not None else None,
                                  _ptr(pos), n_layers, ctypes.byref(cfg) if cfg is not None else None,
                                  order.ctypes.data, score.ctypes.data), "qv2_rank_tensors")
    return order[:n_layers], score[:n_layers]


class PassOutputs:
    """Reusable host-side outputs of qv2_sensitivity_pass for one plan: a pinned mirror of the
    per-tensor records and numpy arrays for the metrics and the list."""

    def __init__(self, plan: "Plan", n_layers: int, device="cuda"):
        import torch
        nt = plan.num_tensors
        self.n_layers = int(n_layers)
        self.n_ts = nt * TENSOR_SUMS.itemsize
        self.d_records = torch.zeros(self.n_ts + nt * PAIR_SUMS.itemsize, dtype=torch.uint8, device=device)
        self.h_records = torch.zeros(self.d_records.shape, dtype=torch.uint8, pin_memory=True)
        self.tensor_sums = self.h_records[:self.n_ts].numpy().view(TENSOR_SUMS)
        self.pair_sums = self.h_records[self.n_ts:].numpy().view(PAIR_SUMS)
        self.metrics = np.zeros(nt, dtype=METRICS)
        self.pair_mse = np.zeros(nt, np.float64)
        self.pair_sqnr_db = np.zeros(nt, np.float64)
        self.order = np.zeros(max(self.n_layers, 1), np.int32)
        self.score = np.zeros(max(self.n_layers, 1), np.float64)


def qv2_sensitivity_pass(plan: "Plan", d_params, d_sums, out: PassOutputs, d_workspace, workspace_bytes=None,
                         stream=None, layer_pos=None, cfg: Optional[qv2_rank_config] = None, strict: bool = True):
    """Steps 1-4 in one native call (synchronises the stream).  Fills `out`; returns (order, score)."""
    w = "qv2_sensitivity_pass"
    ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
    pos = None if layer_pos is None else np.ascontiguousarray(layer_pos, dtype=np.int32)
    if pos is not None and len(pos) != out.n_layers:
        raise QV2Error(QV2_ERR_SHAPE, w)
    need = plan.num_tensors * (TENSOR_SUMS.itemsize + PAIR_SUMS.itemsize)
    if out.h_records.numel() < need or out.metrics.size < plan.num_tensors:
        raise QV2Error(QV2_ERR_SHAPE, f"{w}: outputs made for another plan")
    st = lib().qv2_sensitivity_pass(
        plan.handle, *_seg_args(plan, d_params, d_sums, w), _dev(out.d_records, need, f"{w}: d_records"),
        out.h_records.data_ptr(), ws, wb, _stream(stream), _ptr(pos), out.n_layers,
        ctypes.byref(cfg) if cfg is not None else None, out.metrics.ctypes.data, out.pair_mse.ctypes.data,
        out.pair_sqnr_db.ctypes.data, out.order.ctypes.data, out.score.ctypes.data)
    if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
        raise QV2Error(st, w)
    return out.order[:out.n_layers], out.score[:out.n_layers]


class PreparedPass:
    """qv2_sensitivity_pass (and its two halves) with every argument checked and converted once,
    for callers that run the same pass many times: each call is then one foreign call.
    `outs`: one PassOutputs for run(), two for begin(slot) / end(slot) with two passes in flight."""

    def __init__(self, plan: "Plan", d_params, d_sums, outs, d_workspace, workspace_bytes=None, stream=None,
                 layer_pos=None, cfg: Optional[qv2_rank_config] = None):
        w = "qv2_sensitivity_pass"
        self.plan, self.cfg = plan, cfg
        self.outs = list(outs) if isinstance(outs, (list, tuple)) else [outs]
        ws, wb = _ws(plan, d_workspace, workspace_bytes, w)
        self._keep = (d_params, d_sums, d_workspace)
        self._pos = None if layer_pos is None else np.ascontiguousarray(layer_pos, dtype=np.int32)
        need = plan.num_tensors * (TENSOR_SUMS.itemsize + PAIR_SUMS.itemsize)
        for o in self.outs:
            if o.h_records.numel() < need or o.metrics.size < plan.num_tensors:
                raise QV2Error(QV2_ERR_SHAPE, f"{w}: outputs made for another plan")
            if self._pos is not None and len(self._pos) != o.n_layers:
                raise QV2Error(QV2_ERR_SHAPE, w)
        cfgp = ctypes.byref(cfg) if cfg is not None else None
        st = _stream(stream)
        dev = [(plan.handle, *_seg_args(plan, d_params, d_sums, w), _dev(o.d_records, need, f"{w}: d_records"),
                o.h_records.data_ptr(), ws, wb, st) for o in self.outs]
        host = [(_ptr(self._pos), o.n_layers, cfgp, o.metrics.ctypes.data, o.pair_mse.ctypes.data,
                 o.pair_sqnr_db.ctypes.data, o.order.ctypes.data, o.score.ctypes.data) for o in self.outs]
        self._run = dev[0] + host[0]
        self._begin = [d + (k,) for k, d in enumerate(dev[:2])]
        self._end = [(plan.handle, o.h_records.data_ptr(), k) + h for k, (o, h) in enumerate(zip(self.outs[:2], host))]
        L = lib()
        self._f_run, self._f_begin, self._f_end = L.qv2_sensitivity_pass, L.qv2_sensitivity_pass_begin, \
            L.qv2_sensitivity_pass_end

    def run(self, strict: bool = True):
        st = self._f_run(*self._run)
        if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
            raise QV2Error(st, "qv2_sensitivity_pass")
        return self.outs[0]

    def begin(self, slot: int):
        st = self._f_begin(*self._begin[slot])
        if st != QV2_OK:
            raise QV2Error(st, "qv2_sensitivity_pass_begin")

    def end(self, slot: int, strict: bool = True):
        st = self._f_end(*self._end[slot])
        if st != QV2_OK and (strict or st != QV2_ERR_NONFINITE):
            raise QV2Error(st, "qv2_sensitivity_pass_end")
        return self.outs[slot]


QV2_ORDER_INORDER, QV2_ORDER_WEIGHT_SQNR = 0, 1


def qv2_baseline_order(kind: int, w_sqnr_db=None, n_layers: Optional[int] = None) -> np.ndarray:
    ws = _f64(w_sqnr_db)
    n = len(ws) if n_layers is None else n_layers
    order = np.zeros(max(n, 1), np.int32)
    _check(lib().qv2_baseline_order(kind, _ptr(ws), n, order.ctypes.data), "qv2_baseline_order")
    return order[:n]


def qv2_bops_reduction_pct(macs, keep_fp32) -> float:
    m = _f64(macs)
    k = np.ascontiguousarray(keep_fp32, dtype=np.uint8)
    if len(k) != len(m):
        raise QV2Error(QV2_ERR_SHAPE, "qv2_bops_reduction_pct")
    out = ctypes.c_double()
    _check(lib().qv2_bops_reduction_pct(m.ctypes.data, k.ctypes.data, len(m), ctypes.addressof(out)),
           "qv2_bops_reduction_pct")
    return out.value


def qv2_bops_select(order, macs, target_pct: float):
    """Returns (keep_fp32 flags by layer, number of layers kept, achieved reduction %)."""
    o = np.ascontiguousarray(order, dtype=np.int32)
    m = _f64(macs)
    if len(o) != len(m):
        raise QV2Error(QV2_ERR_SHAPE, "qv2_bops_select")
    keep = np.zeros(max(len(m), 1), np.uint8)
    nk, pct = ctypes.c_int32(), ctypes.c_double()
    _check(lib().qv2_bops_select(o.ctypes.data, m.ctypes.data, len(m), float(target_pct), keep.ctypes.data,
                                 ctypes.addressof(nk), ctypes.addressof(pct)), "qv2_bops_select")
    return keep[:len(m)].astype(bool), nk.value, pct.value


# ----------------------------------------------------------------------------
# convenience: device output buffers for a plan (torch is only the allocator)
# ----------------------------------------------------------------------------
class Buffers:
    def __init__(self, plan: Plan, device="cuda"):
        import torch
        self.params = torch.zeros(plan.num_segments * QPARAMS.itemsize, dtype=torch.uint8, device=device)
        self.sums = torch.zeros(plan.num_segments * SUMS.itemsize, dtype=torch.uint8, device=device)
        self.pair = torch.zeros(plan.num_tensors * PAIR_SUMS.itemsize, dtype=torch.uint8, device=device)
        self.workspace = torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=device)

    def host(self):
        """Blocking copies of the small result records to numpy."""
        return (self.params.cpu().numpy().view(QPARAMS), self.sums.cpu().numpy().view(SUMS),
                self.pair.cpu().numpy().view(PAIR_SUMS))
