"""Seeded synthetic Dense-and-Sparse layers (stand-in for the paper's offline quantiser, Sec. 4.1-4.2).

This module only *produces inputs*: packed b-bit indices, per-row fp16 look-up tables, fp16 CSR
outliers and fp16 activations, with the shapes and structure of the paper's workloads (LLaMA layer
shapes, one table per output channel, ~0.45 % sparse entries with row-skewed counts, App. C).  It
holds none of the inference arithmetic and is shared by the CPU oracle's tests and by the GPU
library's tests and benchmark.  The heavy lifting is in ``sqgen.c`` (C + OpenMP, built with gcc).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sqgen.c")
_LIB = os.path.join(_HERE, "libsqgen.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sqgen.c into libsqgen.so (no -march flags: identical output on every host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, u64, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double
        L.sqgen_weights.argtypes = [i32, i32, u64, vp]; L.sqgen_weights.restype = None
        L.sqgen_x.argtypes = [i32, i32, u64, vp]; L.sqgen_x.restype = None
        L.sqgen_sens.argtypes = [i32, i32, u64, vp]; L.sqgen_sens.restype = None
        L.sqgen_nnz.argtypes = [i32, i32, f64]; L.sqgen_nnz.restype = i64
        L.sqgen_counts_skewed.argtypes = [i32, i32, i64, f64, f64, u64, vp]; L.sqgen_counts_skewed.restype = i32
        L.sqgen_select_global.argtypes = [i32, i32, i64, vp, vp, vp]; L.sqgen_select_global.restype = i32
        L.sqgen_select_rows.argtypes = [i32, i32, vp, vp, vp]; L.sqgen_select_rows.restype = None
        L.sqgen_quantize.argtypes = [i32, i32, i32] + [vp] * 10; L.sqgen_quantize.restype = i32
        L.sqgen_pack.argtypes = [i32, i32, i32, vp, vp]; L.sqgen_pack.restype = i32
        L.sqgen_threads.argtypes = []; L.sqgen_threads.restype = i32
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def layer_seed(base_seed: int, config_id: int, layer_id: int) -> int:
    """Seed of one layer of a multi-layer configuration (plain integer mixing, no hashing library)."""
    z = (base_seed * 0x9E3779B97F4A7C15 + config_id * 0xBF58476D1CE4E5B9 + layer_id * 0x94D049BB133111EB) % (1 << 64)
    z ^= z >> 31
    return z % (1 << 63)


@dataclass
class Layer:
    """One quantised layer: everything the matvec reads.  fp16 arrays are held as uint16 bit patterns."""
    M: int
    N: int
    bits: int
    B: int
    nnz: int
    qidx: np.ndarray            # uint8 [M * N*bits/8]   packed row-major bit streams
    lut: np.ndarray             # uint16 [M, 2^bits]     fp16 bit patterns
    rowptr: np.ndarray          # int32 [M+1]
    cols: np.ndarray            # int32 [nnz]
    vals: np.ndarray            # uint16 [nnz]            fp16 bit patterns
    x: np.ndarray               # uint16 [N, B]           fp16 bit patterns
    seed: int = 0
    frac: float = 0.0
    skew: Optional[tuple] = None
    idx: Optional[np.ndarray] = None    # uint8 [M, N]   (generator's own copy, tests only)
    wgen: Optional[np.ndarray] = None   # float64 [M, N] (generator's own W_eff, tests only)
    w0: Optional[np.ndarray] = None     # uint16 [M, N]  raw fp16 weights before quantisation
    meta: dict = field(default_factory=dict)

    def algorithmic_bytes(self) -> int:
        """Bytes the method must move for one matvec: indices + tables + CSR + x + y."""
        K = 1 << self.bits
        b = self.M * self.N * self.bits // 8 + self.M * K * 2 + self.B * (self.N + self.M) * 2
        if self.nnz > 0:
            b += self.nnz * 6 + (self.M + 1) * 4
        return b


def make_x(N: int, B: int, seed: int) -> np.ndarray:
    x = np.empty((N, B), dtype=np.uint16)
    _load().sqgen_x(N, B, seed, _p(x))
    return x


def make_weights(M: int, N: int, seed: int) -> np.ndarray:
    w = np.empty((M, N), dtype=np.uint16)
    _load().sqgen_weights(M, N, seed, _p(w))
    return w


def make_sens(M: int, N: int, seed: int) -> np.ndarray:
    """Synthetic per-weight sensitivities, uint16 [M, N] (stand-in for the diagonal Fisher information)."""
    s = np.empty((M, N), dtype=np.uint16)
    _load().sqgen_sens(M, N, seed, _p(s))
    return s


def pack(idx: np.ndarray, bits: int) -> np.ndarray:
    """Pack a uint8 index matrix [M, N] into the layer bit-stream format."""
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, N = idx.shape
    q = np.empty(M * N * bits // 8, dtype=np.uint8)
    rc = _load().sqgen_pack(M, N, bits, _p(idx), _p(q))
    if rc != 0:
        raise ValueError(f"N*bits must be a multiple of 8 (rc={rc})")
    return q


def make_layer(M: int, N: int, bits: int, frac: float = 0.0045, skew: Optional[tuple] = None, B: int = 1,
               seed: int = 20230613, keep_debug: bool = False) -> Layer:
    """Generate one layer.

    skew=None      -> sparse set = the nnz largest |w| of the whole matrix.
    skew=(h, s)    -> ceil(h*M) seeded heavy rows hold round(s*nnz) of the entries (e.g. (0.10, 0.50)).
    keep_debug     -> also return the generator's index matrix, its fp64 W_eff and the raw weights.
    """
    L = _load()
    w0 = make_weights(M, N, seed)
    nnz = int(L.sqgen_nnz(M, N, float(frac)))
    counts = np.zeros(M, dtype=np.int32)
    flag = np.zeros((M, N), dtype=np.uint8)
    if nnz > 0:
        if skew is None:
            rc = L.sqgen_select_global(M, N, nnz, _p(w0), _p(counts), _p(flag))
            if rc != 0:
                raise RuntimeError(f"sqgen_select_global failed rc={rc}")
        else:
            rc = L.sqgen_counts_skewed(M, N, nnz, float(skew[0]), float(skew[1]), seed, _p(counts))
            if rc != 0:
                raise RuntimeError(f"sqgen_counts_skewed failed rc={rc}")
            L.sqgen_select_rows(M, N, _p(w0), _p(counts), _p(flag))
    K = 1 << bits
    qidx = np.empty(M * N * bits // 8, dtype=np.uint8)
    lut = np.empty((M, K), dtype=np.uint16)
    rowptr = np.empty(M + 1, dtype=np.int32)
    cols = np.empty(max(nnz, 0), dtype=np.int32)
    vals = np.empty(max(nnz, 0), dtype=np.uint16)
    idx = np.empty((M, N), dtype=np.uint8) if keep_debug else None
    wgen = np.empty((M, N), dtype=np.float64) if keep_debug else None
    rc = L.sqgen_quantize(M, N, bits, _p(w0), _p(flag), _p(counts), _p(qidx), _p(lut), _p(rowptr), _p(cols),
                          _p(vals), _p(idx), _p(wgen))
    if rc != 0:
        raise RuntimeError(f"sqgen_quantize failed rc={rc}")
    x = make_x(N, B, seed ^ 0x5DEECE66D)
    return Layer(M=M, N=N, bits=bits, B=B, nnz=nnz, qidx=qidx, lut=lut, rowptr=rowptr, cols=cols, vals=vals, x=x,
                 seed=seed, frac=frac, skew=skew, idx=idx, wgen=wgen, w0=w0 if keep_debug else None)


def hand_layer(idx: np.ndarray, lut: np.ndarray, bits: int, rowptr=None, cols=None, vals=None, x=None) -> Layer:
    """Wrap hand-made arrays (tests): idx uint8 [M,N], lut fp16 [M,2^bits], CSR and x fp16 [N,B] optional."""
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, N = idx.shape
    lut16 = np.ascontiguousarray(np.asarray(lut, dtype=np.float16)).view(np.uint16).reshape(M, 1 << bits)
    if rowptr is None:
        rowptr = np.zeros(M + 1, dtype=np.int32); cols = np.zeros(0, dtype=np.int32); vals = np.zeros(0, dtype=np.float16)
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    vals16 = np.ascontiguousarray(np.asarray(vals, dtype=np.float16)).view(np.uint16)
    if x is None:
        x = np.ones((N, 1), dtype=np.float16)
    x = np.asarray(x, dtype=np.float16)
    if x.ndim == 1:
        x = x[:, None]
    x16 = np.ascontiguousarray(x).view(np.uint16)
    return Layer(M=M, N=N, bits=bits, B=x16.shape[1], nnz=int(cols.size), qidx=pack(idx, bits), lut=lut16,
                 rowptr=rowptr, cols=cols, vals=vals16, x=x16, idx=idx)


def threads() -> int:
    return int(_load().sqgen_threads())
