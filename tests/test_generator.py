"""Invariants of the synthetic layer generator and of the storage format (no GPU needed)."""
import os

import numpy as np
import pytest

import gen
import oracle
from oracle import numpy_route as nr

LLAMA7B_BLOCK = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
LLAMA13B_BLOCK = [(5120, 5120)] * 4 + [(13824, 5120)] * 2 + [(5120, 13824)]


def storage_bits(M, N, bits, nnz, count_rowptr):
    """closed-form storage of the format: b-bit indices, 2^b fp16 table entries per row, (fp16 value +
    32-bit column) per sparse entry, optional 32-bit row pointers."""
    b = M * N * bits + M * (1 << bits) * 16
    if nnz:
        b += nnz * 48 + ((M + 1) * 32 if count_rowptr else 0)
    return b


def test_average_bits_match_paper_table(golden_dir):
    """P5: format pin — fp16 per-row tables and 48-bit CSR entries reproduce Tab. 1's average bits."""
    for line in open(os.path.join(golden_dir, "paper_avg_bits.txt")):
        if line.startswith("#") or not line.strip():
            continue
        bits, frac, avg_printed, comp_printed = [float(s) for s in line.split("|")]
        bits = int(bits)
        block = LLAMA13B_BLOCK if bits == 2 else LLAMA7B_BLOCK        # the 2-bit lines are the 13B column of App. F
        total_w = sum(M * N for M, N in block)
        for count_rowptr in (False, True):
            tot = sum(storage_bits(M, N, bits, gen._load().sqgen_nnz(M, N, frac), count_rowptr) for M, N in block)
            avg = tot / total_w
            assert abs(avg - avg_printed) < (0.016 if bits == 2 and count_rowptr else 0.011), (bits, frac, avg)
            if bits != 2:                                              # App. F prints no compression rate
                assert abs(16 / avg - comp_printed) < 0.015, (bits, frac, 16 / avg)
        if bits == 2:
            continue
        # alternatives the table rules out: 16-bit columns, fp32 tables
        if frac:
            alt = sum(M * N * bits + M * (1 << bits) * 16 + gen._load().sqgen_nnz(M, N, frac) * 32 for M, N in LLAMA7B_BLOCK) / total_w
            assert abs(alt - avg_printed) > 0.05
        alt = sum(M * N * bits + M * (1 << bits) * 32 for M, N in LLAMA7B_BLOCK) / total_w + frac * 48
        assert abs(alt - avg_printed) > 0.02


def test_algorithmic_bytes_formula():
    L = gen.make_layer(256, 1024, 3, frac=0.0045, skew=(0.1, 0.5))
    assert L.algorithmic_bytes() == 256 * 1024 * 3 // 8 + 256 * 8 * 2 + L.nnz * 6 + 257 * 4 + (1024 + 256) * 2
    # value quoted for the 11008 x 4096 3-bit layer with 0.45 % sparse entries
    nnz = gen._load().sqgen_nnz(11008, 4096, 0.0045)
    assert nnz == 202899
    assert 11008 * 4096 * 3 // 8 + 11008 * 16 + nnz * 6 + 11009 * 4 + (4096 + 11008) * 2 == 18376054


@pytest.mark.parametrize("bits,skew,frac", [(3, (0.1, 0.5), 0.0045), (4, None, 0.0045), (3, (0.01, 0.3), 0.0045),
                                            (4, (0.1, 0.5), 0.01), (3, None, 0.0005), (3, None, 0.0), (2, (0.1, 0.5), 0.0045), (2, None, 0.001)])
def test_layer_invariants(bits, skew, frac):
    M, N = 600, 1024
    L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=1, seed=77, keep_debug=True)
    K = 1 << bits
    # table: M * 2^b entries, strictly ascending, finite
    lut = L.lut.view(np.float16).astype(np.float64)
    assert lut.shape == (M, K) and np.isfinite(lut).all()
    assert (np.diff(lut, axis=1) > 0).all()
    # sparsity level: nnz == round(frac * M * N)
    assert L.nnz == int(round(frac * M * N)) == L.cols.size == L.vals.size
    rp = L.rowptr
    assert rp[0] == 0 and rp[-1] == L.nnz and (np.diff(rp) >= 0).all()
    for i in range(M):
        c = L.cols[rp[i]:rp[i + 1]]
        assert (np.diff(c) > 0).all() and (c >= 0).all() and (c < N).all()
    counts = np.diff(rp)
    if skew and L.nnz:
        nh = int(np.ceil(skew[0] * M - 1e-9))
        heavy = np.sort(counts)[::-1][:nh].sum()
        assert abs(heavy - round(skew[1] * L.nnz)) <= 1
    # indices in range, packed size
    assert L.idx.max() < K and L.qidx.size == M * N * bits // 8
    # reconstruction invariant: unpack -> table -> + scatter(CSR) equals the generator's own W exactly
    assert np.array_equal(oracle.unpack(M, N, bits, L.qidx), L.idx)
    W = nr.dense_weff(M, N, bits, L.qidx, L.lut, L.rowptr, L.cols, L.vals)
    assert np.array_equal(W, L.wgen)
    # sparse values are the original fp16 weights; extracted set = largest magnitudes (per row or global)
    w0 = L.w0.view(np.float16).astype(np.float64)
    rows = np.repeat(np.arange(M), counts)
    assert np.array_equal(L.vals.view(np.float16).astype(np.float64), w0[rows, L.cols])
    mask = np.zeros((M, N), bool); mask[rows, L.cols] = True
    if L.nnz:
        if skew is None:
            assert np.abs(w0[mask]).min() >= np.abs(w0[~mask]).max()
        else:
            for i in np.flatnonzero(counts)[:50]:
                assert np.abs(w0[i][mask[i]]).min() >= np.abs(w0[i][~mask[i]]).max()
    # non-extracted positions hold the nearest centroid; extracted ones the centroid nearest zero
    d = np.abs(w0[:, :, None] - lut[:, None, :])
    near = d.argmin(axis=2)
    assert np.array_equal(L.idx[~mask], near[~mask].astype(np.uint8))
    zero_idx = np.abs(lut).argmin(axis=1)
    assert np.array_equal(L.idx[mask], zero_idx[rows].astype(np.uint8))


def test_generator_is_deterministic_and_seeded():
    a = gen.make_layer(128, 256, 3, seed=1)
    b = gen.make_layer(128, 256, 3, seed=1)
    c = gen.make_layer(128, 256, 3, seed=2)
    assert np.array_equal(a.qidx, b.qidx) and np.array_equal(a.lut, b.lut) and np.array_equal(a.x, b.x)
    assert not np.array_equal(a.qidx, c.qidx)


def test_weight_distribution_is_heavy_tailed():
    """Student-t(4) scaled by 0.02: variance 2*0.02^2, and far heavier tails than a normal (Sec. 4.2: a
    tiny fraction of the weights spans most of the range)."""
    w = gen.make_weights(512, 2048, 3).view(np.float16).astype(np.float64)
    assert abs(np.median(np.abs(w)) / 0.02 - 0.7407) < 0.01          # median |t_4| = 0.7407
    assert 0.8 < np.var(w) / (2 * 0.02 ** 2) < 1.2
    rng99 = np.quantile(np.abs(w), 0.999)
    assert rng99 / np.abs(w).max() < 0.5                              # 99.9 % of the mass in a fraction of the range
    x = gen.make_x(4096, 4, 5).view(np.float16).astype(np.float64)
    assert abs(x.mean()) < 0.05 and abs(x.std() - 1) < 0.05
