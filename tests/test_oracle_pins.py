"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the mistake it is meant to catch.  Citations are to the paper's sections.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import gen
import oracle
from oracle import numpy_route as nr


# ---------------------------------------------------------------- fp16 decoding
def test_half_to_double_matches_numpy_for_every_pattern():
    """own fp16 decoder vs numpy's float16 (an independent implementation), all 65536 patterns."""
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = pats.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(p)) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


# ---------------------------------------------------------------- P1: packing order
def _parse_golden(path):
    cases = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, bits, N, elems, exp = [s.strip() for s in line.split("|")]
        bits, N = int(bits), int(N)
        idx = np.zeros((1, N), dtype=np.uint8)
        if elems == "ramp":
            idx[0] = np.arange(N) % (1 << bits)
        elif elems.startswith("all:"):
            idx[0] = int(elems[4:])
        else:
            for tok in elems.split():
                j, v = tok.split(":")
                idx[0, int(j)] = int(v)
        expected = {int(t.split(":")[0]): int(t.split(":")[1], 16) for t in exp.split()}
        cases.append((name, bits, N, idx, expected))
    return cases


def test_hand_computed_bytes(golden_dir):
    """wrong bit order / field order / word size in the unpacker or the packer."""
    for name, bits, N, idx, expected in _parse_golden(os.path.join(golden_dir, "packing_bytes.txt")):
        # (a) the generator's packer produces the hand-computed bytes
        q = gen.pack(idx, bits)
        for off, byte in expected.items():
            assert q[off] == byte, (name, off, hex(q[off]), hex(byte))
        # (b) the oracle's unpackers read a stream made ONLY from the golden bytes + zeros where the
        #     golden file fully determines it (ramps: rebuild the whole stream from the period)
        if name.startswith("ramp") or name == "all7":
            period = {2: [0xE4], 3: [0x88, 0xC6, 0xFA], 4: [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]}[bits]
            stream = np.array([0xFF] * (N * bits // 8) if name == "all7" else
                              [period[i % len(period)] for i in range(N * bits // 8)], dtype=np.uint8)
        else:
            stream = np.zeros(N * bits // 8, dtype=np.uint8)
            for off, byte in expected.items():
                stream[off] = byte
        assert np.array_equal(oracle.unpack(1, N, bits, stream), idx), name
        assert np.array_equal(nr.unpack(1, N, bits, stream), idx), name


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N", [128, 256, 384, 1024, 4096, 11008])
def test_pack_unpack_roundtrip(bits, N):
    """P2: packer (generator) and the two unpackers (oracle, written separately) are inverse."""
    rng = np.random.default_rng(N * 10 + bits)
    idx = rng.integers(0, 1 << bits, size=(3, N), dtype=np.uint8)
    q = gen.pack(idx, bits)
    assert q.size == 3 * N * bits // 8
    assert np.array_equal(oracle.unpack(3, N, bits, q), idx)
    assert np.array_equal(nr.unpack(3, N, bits, q), idx)


# ---------------------------------------------------------------- P7: exact brute force
def _frac(h):
    return Fraction(float(np.uint16(h).view(np.float16)))


@pytest.mark.parametrize("bits,N,B", [(3, 128, 1), (4, 32, 1), (3, 256, 2), (4, 64, 3), (2, 128, 5), (3, 128, 16)])
def test_bruteforce_exact_rationals(bits, N, B):
    """everything at once on a tiny layer: triple loop in exact rational arithmetic (Sec. 4.2: WX = DX + SX)."""
    M = 4
    rng = np.random.default_rng(7 + bits + N)
    idx = rng.integers(0, 1 << bits, size=(M, N), dtype=np.uint8)
    lut = np.sort(rng.standard_normal((M, 1 << bits)).astype(np.float16), axis=1)
    rowptr = np.array([0, 3, 3, 4, 8], dtype=np.int32)
    cols = np.array([1, 5, N - 1, 0, 2, 3, 9, N - 2], dtype=np.int32)
    vals = (rng.standard_normal(8) * 3).astype(np.float16)
    x = rng.standard_normal((N, B)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    y, a = oracle.layer_matvec(L)
    lut16, vals16, x16 = lut.view(np.uint16), vals.view(np.uint16), x.view(np.uint16)
    for i in range(M):
        for t in range(B):
            s = Fraction(0)
            for j in range(N):
                s += _frac(lut16[i, idx[i, j]]) * _frac(x16[j, t])
            for p in range(rowptr[i], rowptr[i + 1]):
                s += _frac(vals16[p]) * _frac(x16[cols[p], t])
            assert abs(Fraction(float(y[i, t])) - s) <= abs(s) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60), (i, t)
            w = [_frac(lut16[i, idx[i, j]]) for j in range(N)]
            for p in range(rowptr[i], rowptr[i + 1]):
                w[cols[p]] += _frac(vals16[p])
            ad = sum(abs(w[j]) * abs(_frac(x16[j, t])) for j in range(N))
            assert abs(Fraction(float(a[i, t])) - ad) <= ad * Fraction(1, 2 ** 48), (i, t)


# ---------------------------------------------------------------- P3: two routes
@pytest.mark.parametrize("bits,skew,B", [(3, (0.1, 0.5), 2), (4, None, 2), (3, (0.01, 0.3), 2), (2, (0.1, 0.5), 16), (3, None, 11)])
def test_two_oracle_routes_agree(bits, skew, B):
    L = gen.make_layer(384, 1024, bits, frac=0.0045, skew=skew, B=B, seed=11 + bits)
    y, a = oracle.layer_matvec(L)
    y2, a2 = nr.matvec(L.M, L.N, L.bits, L.qidx, L.lut, L.rowptr, L.cols, L.vals, L.x)
    assert np.all(np.abs(y - y2) <= 1e-12 * a2)
    assert np.all(np.abs(a - a2) <= 1e-12 * a2)
    assert np.array_equal(oracle.dequant(L.M, L.N, L.bits, L.qidx, L.lut).view(np.float16).astype(np.float64),
                          nr.dense_weff(L.M, L.N, L.bits, L.qidx, L.lut))


# ---------------------------------------------------------------- P4: special cases -> library / closed forms
def _rand_layer(bits, M=16, N=256, nnz_per_row=4, B=1, seed=0):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, 1 << bits, size=(M, N), dtype=np.uint8)
    lut = np.sort((rng.standard_normal((M, 1 << bits)) * 0.05).astype(np.float16), axis=1)
    cols = np.concatenate([np.sort(rng.choice(N, nnz_per_row, replace=False)) for _ in range(M)]).astype(np.int32)
    rowptr = (np.arange(M + 1) * nnz_per_row).astype(np.int32)
    vals = rng.standard_normal(M * nnz_per_row).astype(np.float16)
    x = rng.standard_normal((N, B)).astype(np.float16)
    return idx, lut, rowptr, cols, vals, x


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_dense_only_reduces_to_numpy_matmul(bits):
    """dropped dense term, wrong table row (table of row i must be used for row i: Sec. 5, one LUT per output channel)."""
    idx, lut, _, _, _, x = _rand_layer(bits, seed=1)
    L = gen.hand_layer(idx, lut, bits, x=x)
    y, _ = oracle.layer_matvec(L)
    W = np.take_along_axis(lut.astype(np.float64), idx.astype(np.int64), axis=1)
    ref = W @ x.astype(np.float64)
    assert np.allclose(y, ref, rtol=0, atol=1e-12)
    # a transposed / shared table would give this instead:
    wrong = np.take_along_axis(np.broadcast_to(lut[0].astype(np.float64), lut.shape), idx.astype(np.int64), axis=1) @ x.astype(np.float64)
    assert not np.allclose(y, wrong, atol=1e-6)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_sparse_only_reduces_to_scipy_csr(bits):
    """CSR semantics: rowptr ranges, column gather, duplicates add (Sec. 4.2: S stored in CSR)."""
    idx, lut, rowptr, cols, vals, x = _rand_layer(bits, seed=2, B=2)
    k0 = 2
    lut = lut.copy(); lut[:, k0] = 0
    idx[:] = k0                                     # dense part is identically zero
    # add a duplicate entry in row 0
    cols = np.concatenate([[cols[0]], cols]).astype(np.int32); vals = np.concatenate([[np.float16(1.5)], vals]).astype(np.float16)
    rowptr = rowptr.copy(); rowptr[1:] += 1
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    y, _ = oracle.layer_matvec(L)
    S = sp.csr_matrix((vals.astype(np.float64), cols, rowptr), shape=idx.shape)   # scipy sums duplicates on use
    assert np.allclose(y, S @ x.astype(np.float64), rtol=0, atol=1e-12)
    y_s, _ = oracle.layer_matvec(L, dense=False)
    assert np.allclose(y_s, y, rtol=0, atol=1e-12)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_identity_table_counts_indices(bits):
    """lut[i][k] = k and x = 1  =>  y_i = sum_j idx_ij exactly (integer)."""
    M, N = 5, 384 if bits == 3 else 96
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 1 << bits, size=(M, N), dtype=np.uint8)
    lut = np.tile(np.arange(1 << bits, dtype=np.float16), (M, 1))
    L = gen.hand_layer(idx, lut, bits)
    y, a = oracle.layer_matvec(L)
    assert np.array_equal(y[:, 0], idx.sum(axis=1).astype(np.float64))
    assert np.array_equal(a, y)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_affine_table_is_uniform_quantisation(bits):
    """lut[i][k] = z_i + s_i k  =>  y_i = z_i sum(x) + s_i sum_j idx_ij x_j (integer matmul identity)."""
    M, N = 6, 256
    rng = np.random.default_rng(4)
    idx = rng.integers(0, 1 << bits, size=(M, N), dtype=np.uint8)
    z = np.array([-2, -1, 0, 1, 2, 3], dtype=np.float64) * 0.25
    s = np.array([1, 2, 0.5, 0.25, 4, 0.125])
    lut = (z[:, None] + s[:, None] * np.arange(1 << bits)).astype(np.float16)      # all exactly representable
    x = rng.integers(-8, 9, size=(N, 1)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, x=x)
    y, _ = oracle.layer_matvec(L)
    xi = x.astype(np.int64)[:, 0]
    ref = z * xi.sum() + s * (idx.astype(np.int64) @ xi)
    assert np.array_equal(y[:, 0], ref)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_unit_vector_extracts_column(bits):
    """x = e_j  =>  y = W_eff[:, j]: catches a wrong column index / off-by-one in either term."""
    idx, lut, rowptr, cols, vals, _ = _rand_layer(bits, seed=5)
    M, N = idx.shape
    W = np.take_along_axis(lut.astype(np.float64), idx.astype(np.int64), axis=1)
    np.add.at(W, (np.repeat(np.arange(M), np.diff(rowptr)), cols), vals.astype(np.float64))
    for j in [0, 1, int(cols[0]), int(cols[-1]), N - 1]:
        x = np.zeros((N, 1), dtype=np.float16); x[j] = 1
        y, a = oracle.layer_matvec(gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x))
        assert np.array_equal(y[:, 0], W[:, j]), j
        assert np.array_equal(a[:, 0], np.abs(W[:, j])), j


def test_sign_and_batch_layout():
    """wrong sign, or x read as [B][N] instead of [N][B]: y(-x) = -y(x); column t of Y depends only on column t of X."""
    idx, lut, rowptr, cols, vals, x = _rand_layer(3, B=3, seed=6)
    L = gen.hand_layer(idx, lut, 3, rowptr, cols, vals, x)
    y, a = oracle.layer_matvec(L)
    yn, an = oracle.layer_matvec(gen.hand_layer(idx, lut, 3, rowptr, cols, vals, -x))
    assert np.array_equal(yn, -y) and np.array_equal(an, a)
    for t in range(3):
        yt, _ = oracle.layer_matvec(gen.hand_layer(idx, lut, 3, rowptr, cols, vals, x[:, t:t + 1]))
        assert np.array_equal(yt[:, 0], y[:, t])


def test_row_range_and_empty_cases():
    idx, lut, rowptr, cols, vals, x = _rand_layer(4, seed=8)
    L = gen.hand_layer(idx, lut, 4, rowptr, cols, vals, x)
    y, _ = oracle.layer_matvec(L)
    yr, _ = oracle.layer_matvec(L, rows=(3, 7))
    assert np.array_equal(yr[3:7], y[3:7]) and np.isnan(yr[:3]).all() and np.isnan(yr[7:]).all()
    # nnz = 0
    L0 = gen.hand_layer(idx, lut, 4, x=x)
    y0, _ = oracle.layer_matvec(L0)
    yd, _ = oracle.layer_matvec(L, sparse=False)
    assert np.array_equal(y0, yd)


# ---------------------------------------------------------------- fp16 baseline oracle
def test_fp16_matvec_is_numpy_matmul():
    rng = np.random.default_rng(9)
    w = rng.standard_normal((7, 96)).astype(np.float16); x = rng.standard_normal((96, 2)).astype(np.float16)
    y, a = oracle.fp16_matvec(w, x)
    assert np.allclose(y, w.astype(np.float64) @ x.astype(np.float64), rtol=0, atol=1e-12)
    assert np.allclose(a, np.abs(w.astype(np.float64)) @ np.abs(x.astype(np.float64)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P8: the tolerance is neither vacuous nor unreachable
def test_tolerance_is_reachable_and_orders_the_accumulators():
    """fp32 accumulation + one fp16 rounding sits far inside 2e-3*absdot (its own bound is 2^-11 |y| +
    N 2^-24 absdot); a running fp16 sum (what Sec. 4.3 describes: all arithmetic in FP16 after
    dequantisation) is an order of magnitude worse, though at these widths still inside the tolerance."""
    L = gen.make_layer(64, 4096, 3, frac=0.0045, skew=(0.1, 0.5), seed=5)
    y, a = oracle.layer_matvec(L)
    W = nr.dense_weff(L.M, L.N, L.bits, L.qidx, L.lut, L.rowptr, L.cols, L.vals)
    xf = L.x.view(np.float16).astype(np.float32)[:, 0]
    acc32 = np.zeros(L.M, dtype=np.float32)
    acc16 = np.zeros(L.M, dtype=np.float16)
    W32 = W.astype(np.float32)
    for j in range(L.N):
        acc32 = acc32 + W32[:, j] * xf[j]
        acc16 = (acc16 + (W32[:, j] * xf[j]).astype(np.float16)).astype(np.float16)
    y32 = acc32.astype(np.float16).astype(np.float64)
    e32 = np.abs(y32 - y[:, 0])
    e16 = np.abs(acc16.astype(np.float64) - y[:, 0])
    assert (e32 <= 2.0 ** -11 * np.abs(y[:, 0]) + L.N * 2.0 ** -24 * a[:, 0]).all()
    assert (e32 / (2e-3 * a[:, 0])).max() < 0.05
    assert e16.mean() > 5 * e32.mean()


# ---------------------------------------------------------------- P2 again, with generated cases
def test_pack_unpack_roundtrip_generated():
    hyp = pytest.importorskip("hypothesis")
    st = pytest.importorskip("hypothesis.strategies")

    @hyp.settings(max_examples=60, deadline=None)
    @hyp.given(bits=st.sampled_from([2, 3, 4]), groups=st.integers(1, 12), rows=st.integers(1, 3), seed=st.integers(0, 2 ** 31 - 1),
               fill=st.sampled_from(["random", "zeros", "max", "alternate"]))
    def check(bits, groups, rows, seed, fill):
        N = 128 * groups
        top = (1 << bits) - 1
        if fill == "random":
            idx = np.random.default_rng(seed).integers(0, top + 1, size=(rows, N), dtype=np.uint8)
        elif fill == "zeros":
            idx = np.zeros((rows, N), dtype=np.uint8)
        elif fill == "max":
            idx = np.full((rows, N), top, dtype=np.uint8)
        else:
            idx = (np.arange(rows * N, dtype=np.int64).reshape(rows, N) % 2 * top).astype(np.uint8)
        q = gen.pack(idx, bits)
        assert q.size == rows * N * bits // 8
        assert np.array_equal(oracle.unpack(rows, N, bits, q), idx)
        assert np.array_equal(nr.unpack(rows, N, bits, q), idx)
        # a single set element changes exactly the bytes its bit field touches
        j = seed % N
        one = np.zeros((1, N), dtype=np.uint8); one[0, j] = top
        touched = np.nonzero(gen.pack(one, bits))[0]
        assert touched.min() == (j * bits) // 8 and touched.max() == (j * bits + bits - 1) // 8

    check()
