"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times
(default rows per workgroup, fused entry point).  Every output row is compared with the CPU oracle; for the
largest shapes the index / dequantisation exports are compared bit-exactly on a band of rows."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3
SEED = 20230613


def run_layer(M, N, bits, frac, skew, B, seed, check_decode_rows=64):
    import paper_2306_07629_amd as sq
    print(f"layer M={M} N={N} bits={bits} frac={frac} skew={skew} B={B} seed={seed}", flush=True)
    L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=B, seed=seed)
    D = sq.DeviceLayer(L)
    y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
    y_ref, absdot = oracle.layer_matvec(L)
    err = np.abs(y - y_ref)
    assert np.isfinite(y).all()
    worst = float(np.max(err / (TOL * absdot)))
    assert worst <= 1.0, f"worst err/bound {worst}"
    tight = 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -24 + (N + 4096) * 2.0 ** -24 * absdot
    assert (err <= tight).all(), float(np.max(err / tight))
    # bit-exact decode on a band of rows in the middle of the matrix (the exports use the same decode code)
    r0 = max(0, M // 2 - check_decode_rows // 2)
    r1 = min(M, r0 + check_decode_rows)
    rb = N * bits // 8
    sub = type("Sub", (), {})()
    sub.M, sub.N, sub.bits, sub.B, sub.nnz = r1 - r0, N, bits, B, 0
    sub.qidx = L.qidx[r0 * rb:r1 * rb]; sub.lut = L.lut[r0:r1]; sub.rowptr = np.zeros(r1 - r0 + 1, np.int32)
    sub.cols = np.zeros(0, np.int32); sub.vals = np.zeros(0, np.uint16); sub.x = L.x
    Ds = sq.DeviceLayer(sub)
    assert np.array_equal(Ds.unpack().cpu().numpy(), oracle.unpack(sub.M, N, bits, sub.qidx))
    assert np.array_equal(Ds.dequantize().cpu().numpy().view(np.uint16), oracle.dequant(sub.M, N, bits, sub.qidx, sub.lut))
    return worst


def test_config1_single_4096_4bit():
    run_layer(4096, 4096, 4, 0.0045, None, 1, gen.layer_seed(SEED, 1, 0), check_decode_rows=4096)


@pytest.mark.parametrize("M,N", [(11008, 4096), (4096, 11008)])
def test_config2_llama7b_mlp_pair_3bit(M, N):
    run_layer(M, N, 3, 0.0045, (0.10, 0.50), 1, gen.layer_seed(SEED, 2, 0 if M > N else 1), check_decode_rows=512)


@pytest.mark.parametrize("M,N", [(5120, 5120), (13824, 5120), (5120, 13824)])
@pytest.mark.parametrize("bits", [3, 4])
def test_config3_llama13b_shapes(M, N, bits):
    run_layer(M, N, bits, 0.0045, None, 1, gen.layer_seed(SEED, 3, M + bits))


@pytest.mark.parametrize("frac", [0.0005, 0.01])
def test_config3_sparsity_sweep(frac):
    run_layer(13824, 5120, 3, frac, None, 1, gen.layer_seed(SEED, 3, int(frac * 1e5)))


def test_config4_one_decoder_block_sequential_on_one_stream():
    """the seven linear layers of one 7B block, fresh seeded weights each, launched back to back"""
    import paper_2306_07629_amd as sq
    shapes = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    layers = [gen.make_layer(M, N, 3, frac=0.0045, skew=(0.10, 0.50), seed=gen.layer_seed(SEED, 4, k)) for k, (M, N) in enumerate(shapes)]
    devs = [sq.DeviceLayer(L) for L in layers]
    for D in devs:              # all seven enqueued before any result is read
        D.matvec()
    for L, D in zip(layers, devs):
        y = D.y_host()
        y_ref, absdot = oracle.layer_matvec(L)
        assert (np.abs(y - y_ref) <= TOL * absdot).all()


@pytest.mark.parametrize("M,N", [(8192, 8192), (22016, 8192), (8192, 22016)])
def test_config5_llama65b_heavy_skew(M, N):
    run_layer(M, N, 3, 0.0045, (0.01, 0.30), 1, gen.layer_seed(SEED, 5, M // 1000 + N // 100))


@pytest.mark.parametrize("B", [2, 4, 8, 16])
def test_config5_batched(B):
    run_layer(8192, 8192, 3, 0.0045, (0.01, 0.30), B, gen.layer_seed(SEED, 5, 100 + B))


@pytest.mark.parametrize("M", [1, 2, 3, 5, 4097])
@pytest.mark.parametrize("bits", [3, 4])
def test_ragged_row_counts(M, bits):
    run_layer(M, 4096, bits, 0.0045, None, 1, 77 + M, check_decode_rows=M)


@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 6, 7, 8, 11, 16])
def test_every_batch_size(B):
    run_layer(70, 2304, 3, 0.0045, (0.1, 0.5), B, 500 + B, check_decode_rows=70)
    run_layer(70, 2304, 4, 0.0045, (0.1, 0.5), B, 600 + B, check_decode_rows=70)


def test_widest_supported_row():
    run_layer(9, 28672, 3, 0.0045, None, 1, 901, check_decode_rows=9)
    run_layer(9, 28672, 4, 0.0045, None, 2, 902, check_decode_rows=9)
    run_layer(9, 28672, 3, 0.0045, None, 16, 903, check_decode_rows=9)
    run_layer(40, 28672, 2, 0.0045, (0.1, 0.5), 9, 904, check_decode_rows=40)


def test_one_row_holds_every_nonzero_of_a_big_block():
    """a row with N nonzeros next to empty rows: exercises the leftover-batch path shared by all waves"""
    import paper_2306_07629_amd as sq
    M, N, bits = 64, 8192, 3
    rng = np.random.default_rng(8)
    idx = rng.integers(0, 8, size=(M, N), dtype=np.uint8)
    lut = np.sort((rng.standard_normal((M, 8)) * 0.05).astype(np.float16), axis=1)
    counts = np.zeros(M, dtype=np.int64); counts[17] = N; counts[18] = 5000; counts[63] = 1
    rowptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    cols = np.concatenate([np.arange(N), np.sort(rng.choice(N, 5000, replace=False)), [N - 1]]).astype(np.int32)
    vals = (rng.standard_normal(cols.size) * 0.1).astype(np.float16)
    x = rng.standard_normal((N, 1)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    y_ref, a_ref = oracle.layer_matvec(L)
    for entry in ("matvec", "csr"):
        D = sq.DeviceLayer(L)
        if entry == "matvec":
            y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
            assert (np.abs(y - y_ref) <= TOL * a_ref).all()
        else:
            ys, as_ = oracle.layer_matvec(L, dense=False)
            y = D.csr_spmv().cpu().numpy().view(np.float16).astype(np.float64)
            assert (np.abs(y - ys) <= TOL * np.maximum(as_, 1e-30)).all()
