"""CPU oracle of the offline side: Dense-and-Sparse split and sensitivity-weighted k-means (paper Sec. 4.1-4.2).

TEST INFRASTRUCTURE ONLY.  Plain numpy / Python integers, one row at a time, written from the paper:

  * Sec. 4.2:  W = D + S with S = W[w < T_min or w > T_max]; the thresholds are percentiles of the weight
    distribution of the matrix.  A small share of highly sensitive weights (largest diagonal Fisher information)
    joins S as well.
  * Sec. 4.1, Eq. 4:  per output channel, Q* = argmin sum_j F_jj (w_j - Q(w_j))^2 over all maps Q onto k = 2^b
    values: a weighted one-dimensional k-means problem.  Solved with Lloyd iterations (the paper names no solver):
    assign every weight to its nearest centroid, move every centroid to the sensitivity-weighted mean of its
    members, repeat.

Lloyd's method is an iteration whose integer decisions (which centroid is nearest) hang on floating point, so this
file fixes the arithmetic of every step and the GPU kernel follows the same steps in the same precision:

  thresholds   order statistics of the monotone 16-bit keys of the fp16 weights / of the 16-bit sensitivities:
               key_min = n_lo-th smallest key, key_max = n_hi-th largest key, s_thr = n_sens-th largest sensitivity
               (0-based); extracted  <=>  key < key_min  or  key > key_max  or  s > s_thr   (strict, so ties stay dense).
  init         c_k = the dense weight of rank floor((2k + 1) n / (2K)) among the row's n dense weights in ascending key
               order (equal-count bins; the paper names no start).  All centroids 0 for a row without dense weights.
  assign       a_j = #{ k < K-1 : fp32(c_k + c_{k+1}) < fp32(2 w_j) }   (nearest centroid, ties to the lower index).
  stop         when no assignment changed since the previous iteration, or after max_iter updates.
  update       S0_k = sum s_j, S1_k = sum s_j * w_j * 2^24 over the members, both exact integers;
               c_k = fp32( fp64(S1_k) * 2^-24 / fp64(S0_k) ), unchanged when S0_k = 0.
  tables       lut_k = fp16(c_k) (round to nearest even); final indices: nearest table entry in exact arithmetic, ties
               to the lower index; an extracted position gets the index of the entry nearest to zero and its full
               fp16 value goes to the CSR matrix.

Parity of the first two pins is bit-exact (indices, tables, CSR arrays).
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------------------------- fp16 helpers
def half_key(bits: np.ndarray) -> np.ndarray:
    """Monotone 16-bit key of fp16 bit patterns: a < b as reals  =>  key(a) < key(b); -0 sorts below +0."""
    b = bits.astype(np.uint16)
    neg = (b & 0x8000) != 0
    return np.where(neg, ~b, b | 0x8000).astype(np.uint16)


def half_to_fixed(bits: np.ndarray) -> np.ndarray:
    """Exact value of finite fp16 bit patterns times 2^24, as int64."""
    b = bits.astype(np.int64)
    e = (b >> 10) & 31
    m = b & 1023
    if np.any(e == 31):
        raise ValueError("non-finite fp16 weight")
    mag = np.where(e == 0, m, (m + 1024) << np.maximum(e - 1, 0))
    return np.where((b & 0x8000) != 0, -mag, mag).astype(np.int64)


def float_to_half_bits(c: np.ndarray) -> np.ndarray:
    """fp32 -> fp16, round to nearest even (numpy's conversion)."""
    return np.asarray(c, dtype=np.float32).astype(np.float16).view(np.uint16)


# ----------------------------------------------------------------------------------------------- Sec. 4.2: the split
def thresholds(w_bits: np.ndarray, sens: np.ndarray, n_lo: int, n_hi: int, n_sens: int):
    """(key_min, key_max, s_thr) as defined in the header."""
    keys = np.sort(half_key(w_bits).ravel())
    ss = np.sort(sens.ravel())
    total = keys.size
    if not (0 <= n_lo < total and 0 <= n_hi < total and 0 <= n_sens < total):
        raise ValueError("counts out of range")
    return int(keys[n_lo]), int(keys[total - 1 - n_hi]), int(ss[total - 1 - n_sens])


def split_mask(w_bits: np.ndarray, sens: np.ndarray, thr) -> np.ndarray:
    key_min, key_max, s_thr = thr
    k = half_key(w_bits)
    return (k < key_min) | (k > key_max) | (sens > s_thr)


def csr_from_mask(w_bits: np.ndarray, mask: np.ndarray):
    M, _ = w_bits.shape
    counts = mask.sum(axis=1)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(counts)
    rows, cols = np.nonzero(mask)          # row-major order: columns ascending within a row
    return rowptr, cols.astype(np.int32), w_bits[rows, cols].astype(np.uint16)


# ----------------------------------------------------------------------------------------------- Sec. 4.1: Lloyd
def _exact_to_f64(hi: int, lo: int) -> np.float64:
    """fp64 of the exact integer hi * 2^32 + lo (|hi| < 2^53, 0 <= lo < 2^53): both terms are exact, one rounding."""
    return np.float64(hi) * np.float64(4294967296.0) + np.float64(lo)


def kmeans_row(w_bits: np.ndarray, sens: np.ndarray, dense: np.ndarray, K: int, max_iter: int):
    """Lloyd iterations on one row.  Returns (centroids fp32 [K], iterations, assignment of the dense entries)."""
    wb = w_bits[dense]
    s = sens[dense].astype(np.int64)
    wf = wb.view(np.float16).astype(np.float32)
    wfix = half_to_fixed(wb)
    c = np.zeros(K, dtype=np.float32)
    if wb.size == 0:
        return c, 0, np.zeros(0, dtype=np.int64)
    order = np.sort(half_key(wb))
    n = wb.size
    for k in range(K):
        key = np.uint16(order[((2 * k + 1) * n) // (2 * K)])
        bits = np.uint16(key & 0x7FFF) if key & 0x8000 else np.uint16(~key)   # inverse of half_key
        c[k] = np.float32(np.array([bits], dtype=np.uint16).view(np.float16)[0])
    two_w = np.float32(2.0) * wf                                  # exact
    p = s * wfix                                                  # |p| < 2^56
    p_lo, p_hi = p & 0xFFFFFFFF, p >> 32                          # p = p_hi * 2^32 + p_lo, 0 <= p_lo < 2^32
    prev = None
    it = 0
    while True:
        t = (c[:-1] + c[1:]).astype(np.float32)
        a = (t[None, :] < two_w[:, None]).sum(axis=1)
        if prev is not None and np.array_equal(a, prev):
            break
        prev = a
        if it == max_iter:
            break
        for k in range(K):
            m = a == k
            s0 = int(s[m].sum())
            if s0 > 0:
                s1 = _exact_to_f64(int(p_hi[m].sum()), int(p_lo[m].sum()))
                c[k] = np.float32(s1 * np.float64(2.0 ** -24) / np.float64(s0))
        it += 1
    return c, it, a


def final_indices(w_bits: np.ndarray, dense: np.ndarray, lut_bits: np.ndarray) -> np.ndarray:
    """Index of the nearest table entry (exact, ties to the lower index); extracted positions: entry nearest to 0."""
    cfix = half_to_fixed(lut_bits)
    wfix = half_to_fixed(w_bits)
    t = cfix[:-1] + cfix[1:]
    idx = (t[None, :] < (2 * wfix)[:, None]).sum(axis=1)
    zero = int(np.argmin(np.abs(cfix)))                           # first minimum = lowest index
    return np.where(dense, idx, zero).astype(np.uint8)


def quantize_layer(w_bits: np.ndarray, sens: np.ndarray, bits: int, n_lo: int, n_hi: int, n_sens: int, max_iter: int = 32,
                   rows=None):
    """The whole offline pass for one matrix.  Returns a dict with idx uint8 [M, N], lut uint16 [M, K], rowptr, cols,
    vals, iters int32 [M] and the thresholds.  `rows` restricts the k-means part to some rows (the split is always
    computed for the whole matrix); idx / lut / iters of the other rows are left zero."""
    M, N = w_bits.shape
    K = 1 << bits
    thr = thresholds(w_bits, sens, n_lo, n_hi, n_sens)
    mask = split_mask(w_bits, sens, thr)
    rowptr, cols, vals = csr_from_mask(w_bits, mask)
    idx = np.zeros((M, N), dtype=np.uint8)
    lut = np.zeros((M, K), dtype=np.uint16)
    iters = np.zeros(M, dtype=np.int32)
    for i in (range(M) if rows is None else rows):
        dense = ~mask[i]
        c, it, _ = kmeans_row(w_bits[i], sens[i], dense, K, max_iter)
        lut[i] = float_to_half_bits(c)
        idx[i] = final_indices(w_bits[i], dense, lut[i])
        iters[i] = it
    return dict(idx=idx, lut=lut, rowptr=rowptr, cols=cols, vals=vals, iters=iters, thresholds=thr, mask=mask)


def objective(w_bits: np.ndarray, sens: np.ndarray, dense: np.ndarray, lut_bits: np.ndarray, idx: np.ndarray):
    """Eq. 4 for one row as an exact integer: sum s_j (w_j - lut[idx_j])^2 * 2^48 over the dense entries."""
    wfix = half_to_fixed(w_bits)
    cfix = half_to_fixed(lut_bits)
    total = 0
    for j in np.nonzero(dense)[0]:
        dlt = int(wfix[j]) - int(cfix[idx[j]])
        total += int(sens[j]) * dlt * dlt
    return total
