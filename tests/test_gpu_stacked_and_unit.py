"""GPU parity for (a) projections that share an input stacked row-wise into one call (exact, because every output row has its
own table -- Sec. 5, quantisation details) and (b) unit-vector inputs, which turn the matvec into an exact read-out of single
weights: y[:, t] must equal fp16(lut[i][idx(i, j)] + S[i][j]) bit for bit, for the one-column kernel and for the 16-column
matrix-core kernel (whose decode path -- entry-major tables, its own field extraction -- no bit-exact export runs through)."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3
SEED = 20230613


def stack(layers):
    """Row-wise concatenation of layers that share N, bits and x: one bigger layer with the rows of all of them."""
    first = layers[0]
    S = type("Stacked", (), {})()
    S.N, S.bits, S.B, S.x = first.N, first.bits, first.B, first.x
    S.M = sum(L.M for L in layers)
    S.qidx = np.concatenate([L.qidx for L in layers])
    S.lut = np.concatenate([L.lut for L in layers])
    S.cols = np.concatenate([L.cols for L in layers])
    S.vals = np.concatenate([L.vals for L in layers])
    rp, base = [np.zeros(1, np.int32)], 0
    for L in layers:
        rp.append(L.rowptr[1:] + base)
        base += int(L.rowptr[-1])
    S.rowptr = np.concatenate(rp).astype(np.int32)
    S.nnz = base
    return S


@pytest.mark.parametrize("parts", [[(4096, 4096)] * 3, [(11008, 4096)] * 2])
def test_stacked_projections_match_the_oracle_and_the_separate_calls(parts):
    """q,k,v -> 12288x4096 and gate,up -> 22016x4096 (3-bit, 0.45 % sparse, 10 % of the rows holding 50 %)"""
    import paper_2306_07629_amd as sq
    print(f"stacked {parts}", flush=True)
    layers = [gen.make_layer(M, N, 3, frac=0.0045, skew=(0.10, 0.50), seed=gen.layer_seed(SEED, 8, k)) for k, (M, N) in enumerate(parts)]
    for L in layers[1:]:
        L.x = layers[0].x                                     # the projections share their input
    S = stack(layers)
    DS = sq.DeviceLayer(S)
    y = DS.matvec().cpu().numpy().copy()
    y_ref, absdot = oracle.layer_matvec(S)
    err = np.abs(y.view(np.float16).astype(np.float64) - y_ref)
    assert (err <= TOL * absdot).all(), float(np.max(err / (TOL * absdot)))
    yd = DS.lut_gemv().cpu().numpy().copy()
    r = 0
    for L in layers:
        D = sq.DeviceLayer(L)
        # the dense term of a row does not depend on which call it belongs to: bit for bit
        assert np.array_equal(D.lut_gemv().cpu().numpy(), yd[r:r + L.M]), "dense term of a stacked row differs from the separate call"
        # with the sparse term the rows of a workgroup share batches of nonzeros, whose boundaries move with the stacking:
        # the fp32 sums may be formed in another order, never by more than the last bits
        ys = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
        diff = np.abs(ys - y[r:r + L.M].view(np.float16).astype(np.float64))
        assert (diff <= 2.0 ** -10 * np.abs(ys) + 2.0 ** -24).all()
        assert (diff == 0).mean() > 0.99
        r += L.M


def expected_column(L, idx, lut_f32, dense_s, j):
    """fp16(fp32(lut[i][idx(i, j)]) + fp32(S[i][j])) for every row i: the one fp32 addition the kernels perform"""
    w = lut_f32[np.arange(L.M), idx[:, j]]
    return (w + dense_s[:, j]).astype(np.float16)


def sparse_as_dense_f32(L):
    S = np.zeros((L.M, L.N), dtype=np.float32)
    rows = np.repeat(np.arange(L.M), np.diff(L.rowptr))
    np.add.at(S, (rows, L.cols), L.vals.view(np.float16).astype(np.float32))
    return S


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M,N", [(70, 384), (8200, 256)])        # 16 and 32 rows per workgroup in the 16-column kernel
def test_unit_vectors_read_out_single_weights_exactly(bits, M, N):
    import torch
    import paper_2306_07629_amd as sq
    print(f"unit vectors bits={bits} M={M} N={N}", flush=True)
    L = gen.make_layer(M, N, bits, frac=0.0045, skew=(0.1, 0.5), B=16, seed=300 + bits + M)
    idx = oracle.unpack(M, N, bits, L.qidx)
    lut_f32 = L.lut.view(np.float16).astype(np.float32)
    Sd = sparse_as_dense_f32(L)
    D = sq.DeviceLayer(L)
    # one 128-column window plus the window boundary: every pair position of a lane's chunk, the pairs straddling 32-bit
    # words, and both halves of a pair
    cols = list(range(128, 256)) + [0, 1, 127, N - 2, N - 1]
    # 16 columns at a time through the matrix-core kernel
    for c0 in range(0, len(cols), 16):
        js = (cols[c0:c0 + 16] + cols[:16])[:16]
        X = np.zeros((N, 16), dtype=np.float16)
        for t, j in enumerate(js):
            X[j, t] = 1.0
        D.x = torch.from_numpy(X.view(np.int16)).cuda()
        y = D.matvec().cpu().numpy().view(np.float16)
        for t, j in enumerate(js):
            want = expected_column(L, idx, lut_f32, Sd, j)
            assert np.array_equal(y[:, t].view(np.uint16), want.view(np.uint16)), f"16-column kernel, column {j}"
    # one column at a time through the vector-ALU kernel (a prefix of the rows keeps the loop short for the tall layer)
    rows = min(M, 70)
    sub = type("Sub", (), {})()
    sub.M, sub.N, sub.bits, sub.B = rows, N, bits, 1
    sub.qidx = L.qidx[:rows * N * bits // 8]; sub.lut = L.lut[:rows]
    sub.rowptr = L.rowptr[:rows + 1].copy(); sub.nnz = int(sub.rowptr[-1])
    sub.cols = L.cols[:sub.nnz]; sub.vals = L.vals[:sub.nnz]
    sub.x = np.zeros((N, 1), dtype=np.uint16)
    D1 = sq.DeviceLayer(sub)
    xs = torch.zeros((len(cols), N), dtype=torch.int16, device="cuda")
    for k, j in enumerate(cols):
        xs[k, j] = 0x3C00                                      # fp16 1.0
    for k, j in enumerate(cols):
        D1.x = xs[k]
        y = D1.matvec().cpu().numpy().view(np.float16)[:, 0]
        want = expected_column(L, idx, lut_f32, Sd, j)[:rows]
        assert np.array_equal(y.view(np.uint16), want.view(np.uint16)), f"one-column kernel, column {j}"
