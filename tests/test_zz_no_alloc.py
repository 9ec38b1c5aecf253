"""The entry point that allocates nothing (sqllm_quantize_layer_noalloc: scratch in a device array of the library) against the
entry point it is a variant of (sqllm_quantize_layer with a caller-owned workspace): every output bit for bit, on two calls
in a row, the second on a smaller input -- the scratch array keeps the first call's contents and must be cleared by the call."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


def run_both(M, N, bits, seed):
    import torch
    import paper_2306_07629_amd as sq
    w, s = gen.make_weights(M, N, seed), gen.make_sens(M, N, seed)
    n_lo, n_hi, n_sens = sq.sqllm_extraction_counts(M, N, 0.004, 0.0005)
    wd = torch.from_numpy(w.view(np.int16)).cuda()
    sd = torch.from_numpy(s.view(np.int16)).cuda()
    ref = sq.quantize_layer(wd, sd, bits, n_lo, n_hi, n_sens, 32)          # existing entry point, workspace from torch
    cap = max(1, n_lo + n_hi + n_sens)
    out = dict(qidx=torch.zeros(M * N * bits // 8, dtype=torch.uint8, device="cuda"), lut=torch.zeros((M, 1 << bits), dtype=torch.int16, device="cuda"),
               rowptr=torch.zeros(M + 1, dtype=torch.int32, device="cuda"), cols=torch.zeros(cap, dtype=torch.int32, device="cuda"),
               vals=torch.zeros(cap, dtype=torch.int16, device="cuda"), iters=torch.zeros(M, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    # every output buffer exists before the call: the call itself must not allocate
    before = torch.cuda.memory_allocated()
    sq.sqllm_quantize_layer_noalloc(M, N, bits, 32, wd, sd, n_lo, n_hi, n_sens, out["qidx"], out["lut"], out["rowptr"], out["cols"], out["vals"], out["iters"])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    nnz = ref.nnz()
    assert int(out["rowptr"][-1].item()) == nnz
    assert torch.equal(out["rowptr"], ref.rowptr) and torch.equal(out["cols"][:nnz], ref.cols[:nnz]) and torch.equal(out["vals"][:nnz], ref.vals[:nnz])
    assert torch.equal(out["lut"], ref.lut) and torch.equal(out["qidx"], ref.qidx) and torch.equal(out["iters"], ref.iters)
    return nnz


def test_no_alloc_entry_point_matches_the_workspace_entry_point_twice_in_a_row():
    print("no-alloc: 300x2048 3-bit, then 70x512 4-bit", flush=True)
    nnz_big = run_both(300, 2048, 3, 11)
    nnz_small = run_both(70, 512, 4, 12)          # smaller input, other table width, same scratch array
    assert nnz_big > nnz_small > 0


def test_no_alloc_entry_point_rejects_what_it_cannot_hold():
    import paper_2306_07629_amd as sq
    A = 1 << 20
    with pytest.raises(sq.SqllmError) as e:
        sq.sqllm_quantize_layer_noalloc(1 << 20, 4096, 3, 8, A, A, 1, 1, 1, A, A, A, A, A, None, stream=0)
    assert "SQLLM_NOALLOC_MAX_WEIGHTS" in str(e.value)
    with pytest.raises(sq.SqllmError):
        sq.sqllm_quantize_layer_noalloc(4, 128, 3, 8, None, A, 1, 1, 1, A, A, A, A, A, None, stream=0)
