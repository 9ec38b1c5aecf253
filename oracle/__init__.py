"""CPU oracle of the Dense-and-Sparse LUT matvec — TEST INFRASTRUCTURE, never part of the product path.

Two independently written routes:
  * ``sqllm_oracle.c``  (this module's ctypes front end): the definition y = D x + S x (Sec. 4.2-4.3) in
    fp64, indices read one bit at a time, OpenMP over rows.  This is the one timed as ``cpu_baseline``.
  * ``oracle.numpy_route``: numpy only — ``unpackbits`` -> indices -> dense fp64 W_eff -> ``W_eff @ x``.
Only tests/, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may import this package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sqllm_oracle.c")
_LIB = os.path.join(_HERE, "libsqoracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _bind(path):
    """ctypes signatures of an oracle library (the default build, or a deliberately broken copy in a test)"""
    if True:
        L = ctypes.CDLL(path)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.orc_half_to_double.argtypes = [ctypes.c_uint16]; L.orc_half_to_double.restype = ctypes.c_double
        L.orc_unpack.argtypes = [i32, i32, i32, vp, vp]; L.orc_unpack.restype = None
        L.orc_dequant.argtypes = [i32, i32, i32, vp, vp, vp]; L.orc_dequant.restype = None
        L.orc_matvec_rows.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp]
        L.orc_matvec_rows.restype = None
        L.orc_fp16_matvec.argtypes = [i32, i32, i32, vp, vp, vp, vp]; L.orc_fp16_matvec.restype = None
        L.orc_threads.argtypes = []; L.orc_threads.restype = i32
    return L


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    return _lib


class use_library:
    """Context manager: route every call of this module through another build of the oracle source
    (tests plant mistakes in a copy of the C file and check that the pins notice)."""

    def __init__(self, path):
        self.path = path

    def __enter__(self):
        global _lib
        self.saved = _lib
        _lib = _bind(self.path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u8(a):
    return np.ascontiguousarray(a).view(np.uint8).reshape(-1)


def _u16(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint16) if a.dtype != np.uint16 else a


def half_to_double(bits: int) -> float:
    return float(_load().orc_half_to_double(int(bits) & 0xFFFF))


def unpack(M, N, bits, qidx) -> np.ndarray:
    """uint8 [M, N]: index of every element (Sec. 4.3: the compressed matrix stores b-bit indices)."""
    out = np.empty((M, N), dtype=np.uint8)
    _load().orc_unpack(M, N, bits, _p(_u8(qidx)), _p(out))
    return out


def dequant(M, N, bits, qidx, lut) -> np.ndarray:
    """uint16 [M, N]: fp16 bit pattern lut[i][idx(i,j)] (Sec. 4.3: indices select fp16 table entries)."""
    out = np.empty((M, N), dtype=np.uint16)
    _load().orc_dequant(M, N, bits, _p(_u8(qidx)), _p(_u16(lut)), _p(out))
    return out


def matvec(M, N, bits, B, qidx, lut, rowptr, cols, vals, x, rows=None, want_absdot=True):
    """(y, absdot), float64 [M, B] each: y = D x + S x (Sec. 4.2) and sum_j |W_eff||x|.

    qidx=None -> sparse term only; rowptr=None or empty cols -> dense term only.
    rows=(r0, r1) restricts the computation to that row range (other rows are NaN).
    """
    y = np.full((M, B), np.nan, dtype=np.float64)
    a = np.full((M, B), np.nan, dtype=np.float64) if want_absdot else None
    r0, r1 = (0, M) if rows is None else rows
    nnz = 0 if (rowptr is None or cols is None) else int(np.asarray(cols).size)
    q = None if qidx is None else _u8(qidx)
    l = None if lut is None else _u16(lut)
    rp = None if nnz == 0 else np.ascontiguousarray(rowptr, dtype=np.int32)
    cl = None if nnz == 0 else np.ascontiguousarray(cols, dtype=np.int32)
    vl = None if nnz == 0 else _u16(vals)
    xx = _u16(x)
    _load().orc_matvec_rows(M, N, bits, B, r0, r1, _p(q), _p(l), nnz, _p(rp), _p(cl), _p(vl), _p(xx), _p(y), _p(a))
    return y, a


def layer_matvec(L, rows=None, dense=True, sparse=True):
    """Oracle result for a generated ``gen.Layer``."""
    return matvec(L.M, L.N, L.bits, L.B, L.qidx if dense else None, L.lut,
                  L.rowptr if sparse else None, L.cols if sparse else None, L.vals if sparse else None, L.x, rows=rows)


def fp16_matvec(w16, x16):
    """fp64 product of an fp16 matrix [M, N] with fp16 activations [N, B]: the plain y = W x."""
    w16 = _u16(w16); x16 = _u16(x16)
    M, N = w16.shape
    B = x16.shape[1]
    y = np.empty((M, B), dtype=np.float64); a = np.empty((M, B), dtype=np.float64)
    _load().orc_fp16_matvec(M, N, B, _p(w16), _p(x16), _p(y), _p(a))
    return y, a


def threads() -> int:
    return int(_load().orc_threads())
