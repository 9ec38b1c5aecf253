"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bars: unpacked indices and dequantised weights bit-exact; y within 2e-3 * sum_j |W_ij||x_j| per element
(and, stricter, within the bound that follows from fp32 accumulation + one fp16 rounding)."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _dev(L):
    import paper_2306_07629_amd as sq
    return sq.DeviceLayer(L)


def check_y(y_gpu, y_ref, absdot, N, what=""):
    err = np.abs(y_gpu - y_ref)
    # results below the fp16 normal range (|y| < 2^-14) are stored on the subnormal grid, whose spacing is 2^-24:
    # half of that is the rounding error of ANY fp16 result there, whatever the arithmetic before it
    bound = TOL * absdot + 2.0 ** -25
    worst = np.max(err / np.maximum(bound, 1e-300))
    assert np.isfinite(y_gpu).all(), what
    assert (err <= bound).all(), f"{what}: worst err/bound = {worst:.3g}"
    # derived bound: half an fp16 ulp of y (normal range) + fp32 accumulation error over N + a few terms
    tight = 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -24 + (N + 64) * 2.0 ** -24 * absdot
    assert (err <= tight).all(), f"{what}: exceeds fp32-accumulation bound by {np.max(err / tight):.3g}"
    return worst


SMALL = [  # (M, N, bits, frac, skew, B)  — several 2048-column slices, ragged last slice, ragged row blocks
    (37, 128, 2, 0.0, None, 1),
    (37, 128, 3, 0.0, None, 1),
    (37, 128, 4, 0.0, None, 1),
    (301, 2176, 2, 0.0045, (0.1, 0.5), 1),
    (130, 4096, 2, 0.001, None, 1),
    (67, 11008, 2, 0.0045, (0.1, 0.5), 1),
    (33, 22016, 2, 0.0045, (0.01, 0.3), 1),
    (65, 8192, 2, 0.0045, (0.01, 0.3), 4),
    (65, 2304, 2, 0.0045, None, 3),
    (301, 2048, 3, 0.0045, (0.1, 0.5), 1),
    (301, 2176, 4, 0.0045, (0.1, 0.5), 1),
    (130, 4096, 3, 0.0045, None, 1),
    (130, 4096, 4, 0.0045, None, 1),
    (67, 5120, 3, 0.01, (0.01, 0.3), 1),
    (67, 11008, 3, 0.0045, (0.1, 0.5), 1),
    (67, 11008, 4, 0.0005, None, 1),
    (33, 22016, 3, 0.0045, (0.01, 0.3), 1),
    (129, 4096, 3, 0.0045, (0.1, 0.5), 2),
    (129, 4096, 4, 0.0045, (0.1, 0.5), 3),
    (65, 8192, 3, 0.0045, (0.01, 0.3), 4),
    (65, 2304, 4, 0.0045, None, 8),
    (65, 2304, 3, 0.0045, None, 5),
    # 5 .. 16 columns (and 3): one launch of the 16-column matrix-core kernel
    (17, 128, 3, 0.0, None, 16),
    (65, 2304, 3, 0.0045, None, 16),
    (65, 2304, 2, 0.0045, (0.1, 0.5), 16),
    (130, 4096, 4, 0.0045, (0.1, 0.5), 12),
    (33, 22016, 3, 0.0045, (0.01, 0.3), 9),
    (301, 2176, 4, 0.01, (0.01, 0.3), 7),
    (129, 1024, 3, 0.0045, (0.1, 0.5), 6),
    (8200, 256, 3, 0.0045, (0.01, 0.3), 16),      # 32 rows per workgroup, ragged last workgroup
    (8209, 128, 4, 0.0045, (0.1, 0.5), 11),
]


@pytest.mark.parametrize("M,N,bits,frac,skew,B", SMALL)
def test_small_layers_all_entry_points(M, N, bits, frac, skew, B):
    print(f"case M={M} N={N} bits={bits} frac={frac} skew={skew} B={B}", flush=True)
    L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=B, seed=1000 + M + N + bits)
    D = _dev(L)
    # indices and dequantised weights: bit-exact
    assert np.array_equal(D.unpack().cpu().numpy(), oracle.unpack(M, N, bits, L.qidx))
    assert np.array_equal(D.dequantize().cpu().numpy().view(np.uint16), oracle.dequant(M, N, bits, L.qidx, L.lut))
    # fused
    y_ref, a_ref = oracle.layer_matvec(L)
    check_y(D.matvec().cpu().numpy().view(np.float16).astype(np.float64), y_ref, a_ref, N, "fused")
    # dense only
    yd, ad = oracle.layer_matvec(L, sparse=False)
    check_y(D.lut_gemv().cpu().numpy().view(np.float16).astype(np.float64), yd, ad, N, "lut_gemv")
    if L.nnz:
        ys, as_ = oracle.layer_matvec(L, dense=False)
        # as_ was computed on the sparse matrix alone
        check_y(D.csr_spmv().cpu().numpy().view(np.float16).astype(np.float64), ys, as_, N, "csr_spmv")
        check_y(D.csr_spmv(rowwise=True).cpu().numpy().view(np.float16).astype(np.float64), ys, as_, N, "csr_rowwise")
        # dense, then the sparse term appended with accumulate: one extra fp16 rounding of the dense part
        D.lut_gemv()
        y2 = D.csr_spmv(accumulate=1).cpu().numpy().view(np.float16).astype(np.float64)
        assert (np.abs(y2 - y_ref) <= TOL * a_ref).all()


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_every_batch_size(bits):
    """B = 1 .. 16 on one small layer: the one-column kernel and every activation path of the 16-column kernel (2 / 4 /
    8 / 12 / 16 columns: vector loads and in-register pairing; any other B: staged as it lies in memory), fused, dense
    only and accumulating."""
    M, N = 45, 384
    for B in range(1, 17):
        print(f"case bits={bits} B={B}", flush=True)
        L = gen.make_layer(M, N, bits, frac=0.01, skew=(0.1, 0.5), B=B, seed=700 + 17 * bits + B)
        D = _dev(L)
        y_ref, a_ref = oracle.layer_matvec(L)
        check_y(D.matvec().cpu().numpy().view(np.float16).astype(np.float64), y_ref, a_ref, N, f"fused B={B}")
        yd, ad = oracle.layer_matvec(L, sparse=False)
        check_y(D.lut_gemv().cpu().numpy().view(np.float16).astype(np.float64), yd, ad, N, f"dense B={B}")
        y2 = D.lut_gemv(accumulate=1).cpu().numpy().view(np.float16).astype(np.float64)
        assert (np.abs(y2 - 2 * yd) <= 2 * TOL * ad + 2.0 ** -24).all(), f"accumulate B={B}"


@pytest.mark.parametrize("M,N,bits,B", [(8200, 128, 2, 8), (8200, 256, 4, 4), (8222, 128, 3, 12), (8193, 128, 3, 13)])
def test_wide_batches_with_32_rows_per_workgroup(M, N, bits, B):
    print(f"case M={M} N={N} bits={bits} B={B}", flush=True)
    L = gen.make_layer(M, N, bits, frac=0.0045, skew=(0.01, 0.3), B=B, seed=4000 + M + bits + B)
    D = _dev(L)
    y_ref, a_ref = oracle.layer_matvec(L)
    check_y(D.matvec().cpu().numpy().view(np.float16).astype(np.float64), y_ref, a_ref, N, "fused")


def test_seeded_random_shapes_and_batches():
    """24 layers drawn from a fixed seed: rows 1..300 (some beyond 8192 for the 32-row workgroups), widths that are
    multiples of 128 up to 3072, every bit width and batch size, sparse fractions 0 .. 2 % with and without row skew."""
    rng = np.random.default_rng(20230613)
    for case in range(24):
        bits = int(rng.integers(2, 5))
        B = int(rng.integers(1, 17))
        N = 128 * int(rng.integers(1, 25))
        M = int(rng.integers(1, 301)) if case % 6 else 8192 + int(rng.integers(1, 40))
        if M > 8192:
            N = 128 * int(rng.integers(1, 3))
        frac = float(rng.choice([0.0, 0.0005, 0.0045, 0.02]))
        skew = [None, (0.1, 0.5), (0.01, 0.3)][int(rng.integers(0, 3))]
        if skew is not None and M < 100:
            skew = None
        print(f"case {case}: M={M} N={N} bits={bits} B={B} frac={frac} skew={skew}", flush=True)
        L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=B, seed=9000 + case)
        D = _dev(L)
        y_ref, a_ref = oracle.layer_matvec(L)
        check_y(D.matvec().cpu().numpy().view(np.float16).astype(np.float64), y_ref, a_ref, N, f"fused case {case}")
        if L.nnz:
            ys, as_ = oracle.layer_matvec(L, dense=False)
            check_y(D.csr_spmv().cpu().numpy().view(np.float16).astype(np.float64), ys, as_, N, f"sparse case {case}")


def test_results_are_reproducible_run_to_run():
    L = gen.make_layer(512, 4096, 3, frac=0.0045, skew=(0.01, 0.3), seed=5)
    D = _dev(L)
    a = D.matvec().cpu().numpy().copy()
    for _ in range(3):
        assert np.array_equal(D.matvec().cpu().numpy(), a)
    # the batched kernels keep a fixed summation order as well (no floating-point atomics anywhere)
    for B in (2, 4, 7, 16):
        Lb = gen.make_layer(300, 2048, 3, frac=0.0045, skew=(0.01, 0.3), B=B, seed=6)
        Db = _dev(Lb)
        a = Db.matvec().cpu().numpy().copy()
        for _ in range(3):
            assert np.array_equal(Db.matvec().cpu().numpy(), a)


def test_degenerate_sparse_patterns():
    """all nonzeros in one row; empty rows around it; a dense row; duplicates."""
    import paper_2306_07629_amd as sq
    M, N, bits = 70, 2048, 3
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 8, size=(M, N), dtype=np.uint8)
    lut = np.sort((rng.standard_normal((M, 8)) * 0.05).astype(np.float16), axis=1)
    counts = np.zeros(M, dtype=np.int64); counts[5] = N; counts[6] = 3; counts[69] = 700
    rowptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    cols = np.concatenate([np.arange(N), [7, 7, 9], np.sort(rng.choice(N, 700, replace=False))]).astype(np.int32)
    vals = rng.standard_normal(cols.size).astype(np.float16)
    x = rng.standard_normal((N, 1)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    D = sq.DeviceLayer(L)
    y_ref, a_ref = oracle.layer_matvec(L)
    # absdot of the oracle merges duplicates before taking |.|; use the looser triangle bound for them
    a_ref[6] += 2 * np.abs(vals.astype(np.float64)[N:N + 2]).sum() * np.abs(x.astype(np.float64)[7])
    err = np.abs(D.matvec().cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
    assert (err <= TOL * a_ref).all()
    ys, as_ = oracle.layer_matvec(L, dense=False)
    as_[6] = a_ref[6]
    err = np.abs(D.csr_spmv().cpu().numpy().view(np.float16).astype(np.float64) - ys)
    assert (err <= TOL * np.maximum(as_, 1e-30)).all()


def test_degenerate_sparse_patterns_with_sixteen_columns():
    """the sparse term of the 16-column kernel: a full row, rows of 1 and 3 nonzeros next to it, empty rows, a heavy
    last row, nonzero counts that are not multiples of 16, duplicates."""
    import paper_2306_07629_amd as sq
    M, N, bits, B = 70, 1024, 3, 16
    rng = np.random.default_rng(31)
    idx = rng.integers(0, 8, size=(M, N), dtype=np.uint8)
    lut = np.sort((rng.standard_normal((M, 8)) * 0.05).astype(np.float16), axis=1)
    counts = np.zeros(M, dtype=np.int64); counts[5] = N; counts[6] = 3; counts[7] = 1; counts[31] = 17; counts[32] = 15; counts[69] = 333
    rowptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    cols = np.concatenate([np.arange(N), [7, 7, 9], [1000], np.sort(rng.choice(N, 17, replace=False)), np.sort(rng.choice(N, 15, replace=False)),
                           np.sort(rng.choice(N, 333, replace=False))]).astype(np.int32)
    vals = rng.standard_normal(cols.size).astype(np.float16)
    x = rng.standard_normal((N, B)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    D = sq.DeviceLayer(L)
    y_ref, a_ref = oracle.layer_matvec(L)
    a_ref[6] += 2 * np.abs(vals.astype(np.float64)[N:N + 2]).sum() * np.abs(x.astype(np.float64)[7])
    err = np.abs(D.matvec().cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
    assert (err <= TOL * a_ref).all()
    # and with the accumulate flag on top of the dense term alone (one more fp16 rounding)
    D.lut_gemv()
    y2 = D.csr_spmv(accumulate=1).cpu().numpy().view(np.float16).astype(np.float64)
    assert (np.abs(y2 - y_ref) <= TOL * a_ref).all()


def test_special_values_in_tables():
    """subnormal, zero and large table entries; identity-like tables give exact integer results."""
    import paper_2306_07629_amd as sq
    M, N = 9, 4096
    rng = np.random.default_rng(4)
    for bits in (3, 4):
        idx = rng.integers(0, 1 << bits, size=(M, N), dtype=np.uint8)
        lut = np.tile(np.arange(1 << bits, dtype=np.float16), (M, 1))
        D = sq.DeviceLayer(gen.hand_layer(idx, lut, bits))
        y = D.lut_gemv().cpu().numpy().view(np.float16).astype(np.float64)[:, 0]
        exact = idx.sum(axis=1).astype(np.float64)
        assert np.array_equal(y, exact.astype(np.float16).astype(np.float64))
        # subnormal entries (below 2^-14) must contribute, not be flushed
        lut = np.tile((np.arange(1 << bits) * 2.0 ** -20).astype(np.float16), (M, 1))
        x = np.full((N, 1), 16.0, dtype=np.float16)
        L = gen.hand_layer(idx, lut, bits, x=x)
        y = sq.DeviceLayer(L).lut_gemv().cpu().numpy().view(np.float16).astype(np.float64)
        y_ref, a_ref = oracle.layer_matvec(L)
        assert (np.abs(y - y_ref) <= 2.0 ** -10 * np.abs(y_ref)).all(), (bits, y[:3], y_ref[:3])


def test_accumulate_flag():
    L = gen.make_layer(100, 2048, 4, frac=0.0045, seed=9)
    D = _dev(L)
    y1 = D.lut_gemv().cpu().numpy().view(np.float16).astype(np.float64)
    y2 = D.lut_gemv(accumulate=1).cpu().numpy().view(np.float16).astype(np.float64)
    yd, ad = oracle.layer_matvec(L, sparse=False)
    assert (np.abs(y2 - 2 * yd) <= 2 * TOL * ad).all()
    assert np.array_equal((y1.astype(np.float32) * 2).astype(np.float16).astype(np.float64), y2)


def test_fp16_gemv_baseline():
    import torch
    import paper_2306_07629_amd as sq
    rng = np.random.default_rng(12)
    for M, N, B in [(300, 4096, 1), (77, 11008, 1), (64, 1024, 4), (50, 2048, 16), (33, 1024, 11)]:
        w = (rng.standard_normal((M, N)) * 0.02).astype(np.float16)
        x = rng.standard_normal((N, B)).astype(np.float16)
        wd = torch.from_numpy(w.view(np.int16)).cuda(); xd = torch.from_numpy(x.view(np.int16)).cuda()
        yd = torch.zeros((M, B), dtype=torch.int16, device="cuda")
        sq.sqllm_fp16_gemv(M, N, B, wd, xd, yd)
        y_ref, a_ref = oracle.fp16_matvec(w, x)
        check_y(yd.cpu().numpy().view(np.float16).astype(np.float64), y_ref, a_ref, N, "fp16_gemv")
