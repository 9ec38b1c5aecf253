"""The pins must notice plausible mistakes.  Each case plants ONE mistake in a copy of the oracle's C source
(on the CPU, never in the GPU path), builds it, and checks that at least one pin of a small battery fails;
the untouched source passes the same battery."""
import os
import subprocess
import tempfile
from fractions import Fraction

import numpy as np
import pytest

import gen
import oracle
from oracle import numpy_route as nr

SRC = os.path.join(os.path.dirname(oracle.__file__), "sqllm_oracle.c")

MUTATIONS = {
    "bit order inside a byte": ("(row[k >> 3] >> (k & 7)) & 1", "(row[k >> 3] >> (7 - (k & 7))) & 1"),
    "bit order inside a field": ("v |= stream_bit(row, j * bits + t) << t;", "v |= stream_bit(row, j * bits + t) << (bits - 1 - t);"),
    "one table for all rows": ("weff[j] = qidx ? orc_half_to_double(lut[(int64_t)i * K +", "weff[j] = qidx ? orc_half_to_double(lut[(int64_t)0 * K +"),
    "sparse term dropped": ("acc += orc_half_to_double(vals[p]) * orc_half_to_double(x[(int64_t)cols[p] * B + t]);",
                            "acc += 0.0 * orc_half_to_double(vals[p]) * orc_half_to_double(x[(int64_t)cols[p] * B + t]);"),
    "x read as [B][N]": ("for (int j = 0; j < N; ++j) acc += weff[j] * orc_half_to_double(x[(int64_t)j * B + t]);",
                         "for (int j = 0; j < N; ++j) acc += weff[j] * orc_half_to_double(x[(int64_t)t * N + j]);"),
    "sign of the dense term": ("for (int j = 0; j < N; ++j) acc += weff[j] *", "for (int j = 0; j < N; ++j) acc -= weff[j] *"),
    "first entry of every CSR row skipped": ("for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p)\n                        acc +=",
                                             "for (int32_t p = rowptr[i] + 1; p < rowptr[i + 1]; ++p)\n                        acc +="),
    "column index off by one": ("orc_half_to_double(x[(int64_t)cols[p] * B + t]);", "orc_half_to_double(x[(int64_t)((cols[p] + 1) % N) * B + t]);"),
    "fp16 subnormals flushed": ("if (expo == 0)        v = (double)frac * 0x1p-24;", "if (expo == 0)        v = 0.0;"),
    "fp16 exponent bias": ("ldexp(1.0, expo - 15)", "ldexp(1.0, expo - 16)"),
    "absdot without the sparse entries": ("weff[cols[p]] += orc_half_to_double(vals[p]);", "weff[cols[p]] += 0.0;"),
    "absdot without |x|": ("a += fabs(weff[j]) * fabs(orc_half_to_double(x[(int64_t)j * B + t]));", "a += fabs(weff[j]) * orc_half_to_double(x[(int64_t)j * B + t]);"),
    "dequant export uses the index as value": ("w_out[(int64_t)i * N + j] = lut[(int64_t)i * K + row_index(qidx + i * row_bytes, bits, j)];",
                                               "w_out[(int64_t)i * N + j] = (uint16_t)row_index(qidx + i * row_bytes, bits, j);"),
}


def battery():
    """a fast subset of the pins in test_oracle_pins.py; raises AssertionError on the first mismatch"""
    # fp16 decoding, a sample of patterns including subnormals
    for p in (0x0001, 0x03FF, 0x0400, 0x3C00, 0xBC00, 0x7BFF, 0x8001, 0x2E66):
        assert oracle.half_to_double(p) == float(np.uint16(p).view(np.float16)), hex(p)
    # hand-computed packing bytes
    ramp3 = np.array([0x88, 0xC6, 0xFA] * 16, dtype=np.uint8)
    assert np.array_equal(oracle.unpack(1, 128, 3, ramp3)[0], np.arange(128) % 8)
    edge = np.zeros(48, dtype=np.uint8); edge[3] = 0xC0; edge[4] = 0x01
    want = np.zeros(128, dtype=np.uint8); want[10] = 7
    assert np.array_equal(oracle.unpack(1, 128, 3, edge)[0], want)
    nib = np.zeros(16, dtype=np.uint8); nib[1] = 0xC3
    want4 = np.zeros(32, dtype=np.uint8); want4[2] = 3; want4[3] = 12
    assert np.array_equal(oracle.unpack(1, 32, 4, nib)[0], want4)
    # exact rationals on a tiny hand-made layer with a batch of 2 and subnormal table entries
    rng = np.random.default_rng(5)
    M, N, B, bits = 3, 128, 2, 3
    idx = rng.integers(0, 8, size=(M, N), dtype=np.uint8)
    lut = np.sort(rng.standard_normal((M, 8)).astype(np.float16), axis=1)
    lut[1, 3] = np.float16(3e-6)
    rowptr = np.array([0, 2, 2, 5], dtype=np.int32)
    cols = np.array([0, 7, 3, 64, 127], dtype=np.int32)
    vals = np.array([2.5, -1.25, 0.75, 3.0, -0.5], dtype=np.float16)
    x = rng.standard_normal((N, B)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    y, a = oracle.layer_matvec(L)
    fr = lambda v: Fraction(float(v))
    for i in range(M):
        for t in range(B):
            w = [fr(lut[i, idx[i, j]]) for j in range(N)]
            s = sum(w[j] * fr(x[j, t]) for j in range(N))
            for p in range(rowptr[i], rowptr[i + 1]):
                s += fr(vals[p]) * fr(x[cols[p], t]); w[cols[p]] += fr(vals[p])
            ad = sum(abs(w[j]) * abs(fr(x[j, t])) for j in range(N))
            assert abs(fr(y[i, t]) - s) <= abs(s) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 60)
            assert abs(fr(a[i, t]) - ad) <= ad * Fraction(1, 2 ** 45)
    assert np.array_equal(oracle.dequant(M, N, bits, L.qidx, L.lut).view(np.float16), np.take_along_axis(lut, idx.astype(np.int64), axis=1))
    # second route on a generated layer
    G = gen.make_layer(96, 256, 4, frac=0.01, skew=(0.1, 0.5), B=2, seed=3)
    y, a = oracle.layer_matvec(G)
    y2, a2 = nr.matvec(G.M, G.N, G.bits, G.qidx, G.lut, G.rowptr, G.cols, G.vals, G.x)
    assert np.all(np.abs(y - y2) <= 1e-12 * a2) and np.all(np.abs(a - a2) <= 1e-12 * a2)


def build_variant(text, tmpdir, name):
    c = os.path.join(tmpdir, name + ".c"); so = os.path.join(tmpdir, name + ".so")
    open(c, "w").write(text)
    subprocess.run(["gcc", "-O1", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", so, c, "-lm"], check=True)
    return so


def test_untouched_oracle_passes_the_battery():
    battery()
    with tempfile.TemporaryDirectory() as d:
        with oracle.use_library(build_variant(open(SRC).read(), d, "plain")):
            battery()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_noticed(name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target not found in the oracle source: {old!r}"
    with tempfile.TemporaryDirectory() as d:
        so = build_variant(text.replace(old, new), d, "mutant")
        with oracle.use_library(so):
            with pytest.raises(AssertionError):
                battery()
