"""ctypes binding of the C ABI in include/sqllm.h.  Argument marshalling only: every step of the matvec
runs in the HIP kernels of libsqllm.so.  PyTorch tensors are used as owners of device memory and for the
current HIP stream, nothing else.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import sys

from . import build as _build

_lib = None

OK = 0
STATUS_NAMES = ["SQLLM_OK", "SQLLM_ERR_NULL", "SQLLM_ERR_BITS", "SQLLM_ERR_SHAPE", "SQLLM_ERR_ALIGN", "SQLLM_ERR_NNZ",
                "SQLLM_ERR_BATCH", "SQLLM_ERR_HIP", "SQLLM_ERR_DEVICE"]

EXPORTS = ["sqllm_lut_gemv", "sqllm_csr_spmv", "sqllm_dense_sparse_matvec", "sqllm_dense_sparse_matvec_multi", "sqllm_multi_launch_order", "sqllm_csr_spmv_rowwise",
           "sqllm_csr_plan_bytes", "sqllm_csr_plan_build",
           "sqllm_unpack_indices", "sqllm_dequantize", "sqllm_fp16_gemv", "sqllm_algorithmic_bytes",
           "sqllm_quantize_workspace_bytes", "sqllm_quantize_layer", "sqllm_quantize_layer_noalloc", "sqllm_extraction_counts",
           "sqllm_last_error_string", "sqllm_status_string", "sqllm_version"]


class LayerDesc(ctypes.Structure):
    """sqllm_layer of include/sqllm.h"""
    _fields_ = [("M", ctypes.c_int), ("N", ctypes.c_int), ("bits", ctypes.c_int), ("nnz", ctypes.c_longlong),
                ("qidx", ctypes.c_void_p), ("lut", ctypes.c_void_p), ("rowptr", ctypes.c_void_p), ("cols", ctypes.c_void_p),
                ("vals", ctypes.c_void_p), ("plan", ctypes.c_void_p), ("x", ctypes.c_void_p), ("y", ctypes.c_void_p)]


class SqllmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libsqllm.so (built in-tree by build.py).  A missing library, or one older than its sources, is built first."""
    global _lib
    if _lib is None:
        if _build.is_stale():
            print("paper_2306_07629_amd: libsqllm.so is missing or older than its sources, building it", file=sys.stderr, flush=True)
            _build.build()
        L = ctypes.CDLL(_build.LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        L.sqllm_lut_gemv.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
        L.sqllm_csr_spmv.argtypes = [i32, i32, i64, i32, vp, vp, vp, vp, vp, i32, vp]
        L.sqllm_csr_spmv_rowwise.argtypes = [i32, i32, i64, i32, vp, vp, vp, vp, vp, i32, vp]
        L.sqllm_dense_sparse_matvec.argtypes = [i32, i32, i32, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.sqllm_csr_plan_bytes.argtypes = [i32, i32, i64, ctypes.POINTER(ctypes.c_size_t)]
        L.sqllm_csr_plan_build.argtypes = [i32, i32, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.sqllm_dense_sparse_matvec_multi.argtypes = [i32, ctypes.POINTER(LayerDesc), vp]
        L.sqllm_multi_launch_order.argtypes = [i32, ctypes.POINTER(LayerDesc), ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.sqllm_unpack_indices.argtypes = [i32, i32, i32, vp, vp, vp]
        L.sqllm_dequantize.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        L.sqllm_fp16_gemv.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        L.sqllm_algorithmic_bytes.argtypes = [i32, i32, i32, i64, i32]
        L.sqllm_algorithmic_bytes.restype = i64
        L.sqllm_quantize_workspace_bytes.argtypes = [i32, i32]
        L.sqllm_quantize_workspace_bytes.restype = i64
        L.sqllm_quantize_layer.argtypes = [i32, i32, i32, i32, vp, vp, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp]
        L.sqllm_quantize_layer_noalloc.argtypes = [i32, i32, i32, i32, vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp]
        L.sqllm_extraction_counts.argtypes = [i32, i32, ctypes.c_double, ctypes.c_double, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.sqllm_last_error_string.restype = ctypes.c_char_p
        L.sqllm_status_string.argtypes = [i32]
        L.sqllm_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status: int):
    if status != OK:
        raise SqllmError(status, lib().sqllm_last_error_string().decode())


def _ptr(t):
    """Device (or raw integer) pointer of a tensor; None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def sqllm_lut_gemv(M, N, bits, B, qidx, lut, x, y, accumulate=0, stream=None):
    _check(lib().sqllm_lut_gemv(M, N, bits, B, _ptr(qidx), _ptr(lut), _ptr(x), _ptr(y), int(accumulate), _stream(stream)))


def sqllm_csr_spmv(M, N, nnz, B, rowptr, cols, vals, x, y, accumulate=0, stream=None):
    _check(lib().sqllm_csr_spmv(M, N, nnz, B, _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(x), _ptr(y), int(accumulate), _stream(stream)))


def sqllm_csr_spmv_rowwise(M, N, nnz, B, rowptr, cols, vals, x, y, accumulate=0, stream=None):
    _check(lib().sqllm_csr_spmv_rowwise(M, N, nnz, B, _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(x), _ptr(y), int(accumulate), _stream(stream)))


def sqllm_dense_sparse_matvec(M, N, bits, nnz, B, qidx, lut, rowptr, cols, vals, x, y, stream=None, plan=None):
    _check(lib().sqllm_dense_sparse_matvec(M, N, bits, nnz, B, _ptr(qidx), _ptr(lut), _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(plan),
                                           _ptr(x), _ptr(y), _stream(stream)))


def sqllm_csr_plan_bytes(M, N, nnz) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sqllm_csr_plan_bytes(int(M), int(N), int(nnz), ctypes.byref(n)))
    return int(n.value)


def sqllm_csr_plan_build(M, N, nnz, rowptr, cols, vals, plan, nbytes, stream=None):
    _check(lib().sqllm_csr_plan_build(int(M), int(N), int(nnz), _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(plan), int(nbytes), _stream(stream)))


def _addr(t):
    if t is None:
        return None
    return t if isinstance(t, int) else t.data_ptr()


def layer_descriptors(layers):
    """ctypes array of sqllm_layer from (M, N, bits, nnz, qidx, lut, rowptr, cols, vals, x, y[, plan]) tuples (tensors or raw
    addresses)"""
    arr = (LayerDesc * len(layers))()
    for d, t in zip(arr, layers):
        M, N, bits, nnz, qidx, lut, rowptr, cols, vals, x, y = t[:11]
        d.M, d.N, d.bits, d.nnz = M, N, bits, nnz
        d.qidx, d.lut, d.rowptr, d.cols, d.vals, d.x, d.y = (_addr(v) for v in (qidx, lut, rowptr, cols, vals, x, y))
        d.plan = _addr(t[11]) if len(t) > 11 else None
    return arr


def sqllm_dense_sparse_matvec_multi(layers, stream=None):
    """layers: a ctypes array from layer_descriptors(), or the list of tuples it takes"""
    arr = layers if isinstance(layers, ctypes.Array) else layer_descriptors(layers)
    _check(lib().sqllm_dense_sparse_matvec_multi(len(arr), arr, _stream(stream)))


def sqllm_multi_launch_order(layers):
    """(launch number per layer, rows per workgroup per layer, number of launches) of sqllm_dense_sparse_matvec_multi(layers)"""
    arr = layers if isinstance(layers, ctypes.Array) else layer_descriptors(layers)
    n = len(arr)
    launch, rows, total = (ctypes.c_int * max(n, 1))(), (ctypes.c_int * max(n, 1))(), ctypes.c_int(0)
    _check(lib().sqllm_multi_launch_order(n, arr, launch, rows, ctypes.byref(total)))
    return list(launch[:n]), list(rows[:n]), total.value


def sqllm_unpack_indices(M, N, bits, qidx, idx_out, stream=None):
    _check(lib().sqllm_unpack_indices(M, N, bits, _ptr(qidx), _ptr(idx_out), _stream(stream)))


def sqllm_dequantize(M, N, bits, qidx, lut, w_out, stream=None):
    _check(lib().sqllm_dequantize(M, N, bits, _ptr(qidx), _ptr(lut), _ptr(w_out), _stream(stream)))


def sqllm_fp16_gemv(M, N, B, w, x, y, stream=None):
    _check(lib().sqllm_fp16_gemv(M, N, B, _ptr(w), _ptr(x), _ptr(y), _stream(stream)))


def sqllm_quantize_workspace_bytes(M, N) -> int:
    return int(lib().sqllm_quantize_workspace_bytes(M, N))


def sqllm_quantize_layer(M, N, bits, max_iter, w, sens, n_lo, n_hi, n_sens, workspace, workspace_bytes,
                         qidx, lut, rowptr, cols, vals, iters=None, stream=None):
    _check(lib().sqllm_quantize_layer(M, N, bits, max_iter, _ptr(w), _ptr(sens), n_lo, n_hi, n_sens, _ptr(workspace), workspace_bytes,
                                      _ptr(qidx), _ptr(lut), _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(iters), _stream(stream)))


def sqllm_quantize_layer_noalloc(M, N, bits, max_iter, w, sens, n_lo, n_hi, n_sens, qidx, lut, rowptr, cols, vals, iters=None, stream=None):
    _check(lib().sqllm_quantize_layer_noalloc(M, N, bits, max_iter, _ptr(w), _ptr(sens), n_lo, n_hi, n_sens,
                                              _ptr(qidx), _ptr(lut), _ptr(rowptr), _ptr(cols), _ptr(vals), _ptr(iters), _stream(stream)))


def sqllm_algorithmic_bytes(M, N, bits, nnz, B) -> int:
    return int(lib().sqllm_algorithmic_bytes(M, N, bits, nnz, B))


def sqllm_extraction_counts(M, N, outlier_frac, sens_frac):
    n = [ctypes.c_longlong(0) for _ in range(3)]
    _check(lib().sqllm_extraction_counts(int(M), int(N), float(outlier_frac), float(sens_frac), *[ctypes.byref(v) for v in n]))
    return tuple(int(v.value) for v in n)


def sqllm_version() -> int:
    return int(lib().sqllm_version())
