"""GPU parity of the offline entry point (sqllm_quantize_layer, through the C ABI) against the quantiser oracle.

Everything the entry point writes is an integer or a bit pattern decided in fixed precision, so the bar is
bit-exact: CSR arrays, fp16 tables, indices (unpacked by the matvec oracle's bit-at-a-time unpacker) and the number
of centroid updates per row."""
import numpy as np
import pytest

import gen
import oracle
from oracle import quant_oracle as qo

pytestmark = pytest.mark.gpu


def run_gpu(w, s, bits, n_lo, n_hi, n_sens, max_iter):
    import torch
    import paper_2306_07629_amd as sq
    wd = torch.from_numpy(w.view(np.int16)).cuda()
    sd = torch.from_numpy(s.view(np.int16)).cuda()
    q = sq.quantize_layer(wd, sd, bits, n_lo, n_hi, n_sens, max_iter)
    torch.cuda.synchronize()
    nnz = q.nnz()
    return dict(qidx=q.qidx.cpu().numpy(), lut=q.lut.cpu().numpy().view(np.uint16), rowptr=q.rowptr.cpu().numpy(),
                cols=q.cols.cpu().numpy()[:nnz], vals=q.vals.cpu().numpy().view(np.uint16)[:nnz], iters=q.iters.cpu().numpy(), dev=q)


def compare(M, N, bits, got, ref, rows=None):
    assert np.array_equal(got["rowptr"], ref["rowptr"])
    assert np.array_equal(got["cols"], ref["cols"])
    assert np.array_equal(got["vals"], ref["vals"])
    idx = oracle.unpack(M, N, bits, got["qidx"])
    sel = slice(None) if rows is None else rows
    assert np.array_equal(got["iters"][sel], ref["iters"][sel])
    assert np.array_equal(got["lut"][sel], ref["lut"][sel])
    assert np.array_equal(idx[sel], ref["idx"][sel])


CASES = [  # (M, N, bits, outlier_frac, sens_frac, max_iter)
    (33, 128, 2, 0.001, 0.0005, 20),
    (50, 4096, 2, 0.0005, 0.0005, 40),      # the 2-bit + 0.1 % setting of App. F
    (33, 128, 3, 0.0, 0.0, 20),
    (33, 128, 4, 0.004, 0.0005, 20),
    (70, 512, 3, 0.004, 0.0005, 50),
    (70, 640, 4, 0.01, 0.002, 50),
    (40, 4096, 3, 0.004, 0.0005, 40),
    (24, 4096, 4, 0.004, 0.0005, 3),        # stops on the iteration bound
    (12, 11008, 3, 0.004, 0.0005, 40),
    (6, 28672, 4, 0.004, 0.0005, 25),       # widest row the library accepts
    (16, 2304, 3, 0.05, 0.01, 0),           # no updates at all: tables are the equal-count start
]


@pytest.mark.parametrize("M,N,bits,of,sf,max_iter", CASES)
def test_quantize_matches_the_oracle(M, N, bits, of, sf, max_iter):
    import paper_2306_07629_amd as sq
    print(f"case M={M} N={N} bits={bits} outliers={of} sensitive={sf} max_iter={max_iter}", flush=True)
    w = gen.make_weights(M, N, 500 + M + N)
    s = gen.make_sens(M, N, 500 + M + N)
    n_lo, n_hi, n_sens = sq.sqllm_extraction_counts(M, N, of, sf)
    ref = qo.quantize_layer(w, s, bits, n_lo, n_hi, n_sens, max_iter)
    got = run_gpu(w, s, bits, n_lo, n_hi, n_sens, max_iter)
    compare(M, N, bits, got, ref)
    assert got["rowptr"][-1] <= n_lo + n_hi + n_sens


def test_unweighted_and_degenerate_inputs():
    import paper_2306_07629_amd as sq
    M, N, bits = 20, 256, 3
    w = gen.make_weights(M, N, 77)
    ones = np.ones((M, N), dtype=np.uint16)
    # all sensitivities equal: plain k-means (Eq. 1); no weight can be above the sensitivity threshold
    n_lo, n_hi, _ = sq.sqllm_extraction_counts(M, N, 0.01, 0.0)
    compare(M, N, bits, run_gpu(w, ones, bits, n_lo, n_hi, 5, 30), qo.quantize_layer(w, ones, bits, n_lo, n_hi, 5, 30))
    # rows of equal weights, of zeros (both signs), and rows whose sensitivities are all zero
    w2 = w.copy()
    w2[0, :] = np.float16(0.125).view(np.uint16)
    w2[1, :] = 0
    w2[2, ::2] = 0x8000
    w2[2, 1::2] = 0
    s2 = gen.make_sens(M, N, 78)
    s2[3, :] = 0
    s2[4, : N // 2] = 0
    compare(M, N, bits, run_gpu(w2, s2, bits, 3, 3, 3, 30), qo.quantize_layer(w2, s2, bits, 3, 3, 3, 30))
    # a few distinct values only (ties everywhere), 4-bit tables with more entries than values
    rng = np.random.default_rng(9)
    w3 = np.float16(rng.integers(-3, 4, (M, N)) * 0.01).view(np.uint16)
    compare(M, N, 4, run_gpu(w3, s2, 4, 0, 0, 0, 30), qo.quantize_layer(w3, s2, 4, 0, 0, 0, 30))


def test_full_size_layer_on_sampled_rows():
    """LLaMA-7B attention projection (4096 x 4096, 3-bit, 0.4 % outliers + 0.05 % sensitive): the split is checked
    in full, tables / indices / iteration counts on a sample of rows the oracle can afford."""
    import paper_2306_07629_amd as sq
    M, N, bits = 4096, 4096, 3
    w = gen.make_weights(M, N, 4096)
    s = gen.make_sens(M, N, 4096)
    n_lo, n_hi, n_sens = sq.sqllm_extraction_counts(M, N, 0.004, 0.0005)
    rows = np.unique(np.concatenate([[0, 1, M - 1], np.random.default_rng(3).integers(0, M, 45)]))
    ref = qo.quantize_layer(w, s, bits, n_lo, n_hi, n_sens, 40, rows=rows)
    got = run_gpu(w, s, bits, n_lo, n_hi, n_sens, 40)
    compare(M, N, bits, got, ref, rows=rows)
    # properties that hold for every row: ascending tables, indices in range, extracted positions point at the entry
    # nearest to zero
    lut = got["lut"].view(np.float16).astype(np.float64)
    assert np.all(np.diff(lut, axis=1) >= 0)
    assert got["iters"].min() >= 1 and got["iters"].max() <= 40


def test_quantised_layer_runs_through_the_matvec():
    """The entry point's outputs, still on the device, are a valid input of the matvec; the product agrees with the
    matvec oracle evaluated on the same arrays."""
    import torch
    import paper_2306_07629_amd as sq
    M, N, bits = 300, 4096, 4
    w = gen.make_weights(M, N, 91)
    s = gen.make_sens(M, N, 91)
    n_lo, n_hi, n_sens = sq.sqllm_extraction_counts(M, N, 0.004, 0.0005)
    got = run_gpu(w, s, bits, n_lo, n_hi, n_sens, 30)
    q = got["dev"]
    x = gen.make_x(N, 1, 91)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    yd = torch.empty((M, 1), dtype=torch.int16, device="cuda")
    nnz = int(got["rowptr"][-1])
    sq.sqllm_dense_sparse_matvec(M, N, bits, nnz, 1, q.qidx, q.lut, q.rowptr, q.cols, q.vals, xd, yd)
    torch.cuda.synchronize()
    y = yd.cpu().numpy().view(np.float16).astype(np.float64)
    y_ref, absdot = oracle.matvec(M, N, bits, 1, got["qidx"], got["lut"], got["rowptr"], got["cols"], got["vals"], x)
    assert (np.abs(y - y_ref) <= 2e-3 * absdot).all()
    # and the quantised layer is a fair stand-in for the fp16 one: relative error of the product well below one
    y16, _ = oracle.fp16_matvec(w, x)
    assert np.linalg.norm(y_ref - y16) < 0.2 * np.linalg.norm(y16)


def test_argument_errors_do_not_launch():
    import torch
    import paper_2306_07629_amd as sq
    M, N = 8, 128
    w = torch.zeros((M, N), dtype=torch.int16, device="cuda")
    with pytest.raises(sq.SqllmError):
        sq.quantize_layer(w, w, 5, 0, 0, 0)
    with pytest.raises(sq.SqllmError):
        sq.quantize_layer(w, w, 3, M * N, 0, 0)
    with pytest.raises(sq.SqllmError):
        sq.quantize_layer(w, w, 3, 0, 0, 0, max_iter=-1)
