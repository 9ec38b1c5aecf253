"""Second, independently written oracle route (numpy only) — TEST INFRASTRUCTURE.

Materialises W_eff = D + S densely in fp64 and calls ``W_eff @ x`` (Sec. 4.2: W X = D X + S X).
The index matrix is recovered with ``numpy.unpackbits`` on the little-endian bit stream of each row
(element j = stream bits [j*b, j*b+b), least significant first), then the table is applied with
``take_along_axis`` (Sec. 4.3: indices select fp16 table entries; one table per output row, Sec. 5).
"""
from __future__ import annotations

import numpy as np


def unpack(M: int, N: int, bits: int, qidx: np.ndarray) -> np.ndarray:
    stream = np.unpackbits(np.ascontiguousarray(qidx).view(np.uint8).reshape(M, N * bits // 8), axis=1, bitorder="little")
    fields = stream.reshape(M, N, bits).astype(np.uint8)
    weights = (1 << np.arange(bits, dtype=np.uint8)).astype(np.uint8)
    return (fields * weights).sum(axis=2, dtype=np.uint8)


def dense_weff(M, N, bits, qidx, lut, rowptr=None, cols=None, vals=None) -> np.ndarray:
    """float64 [M, N]: lut[i][idx] plus the scattered CSR entries (duplicates add)."""
    lut_f = np.ascontiguousarray(lut).view(np.float16).reshape(M, 1 << bits).astype(np.float64)
    W = np.take_along_axis(lut_f, unpack(M, N, bits, qidx).astype(np.int64), axis=1)
    if cols is not None and np.asarray(cols).size:
        rp = np.asarray(rowptr, dtype=np.int64)
        r = np.repeat(np.arange(M), np.diff(rp))
        v = np.ascontiguousarray(vals).view(np.float16).astype(np.float64)
        np.add.at(W, (r, np.asarray(cols, dtype=np.int64)), v)
    return W


def matvec(M, N, bits, qidx, lut, rowptr, cols, vals, x):
    """(y, absdot) float64 [M, B]."""
    W = dense_weff(M, N, bits, qidx, lut, rowptr, cols, vals)
    xf = np.ascontiguousarray(x).view(np.float16).astype(np.float64).reshape(N, -1)
    return W @ xf, np.abs(W) @ np.abs(xf)
