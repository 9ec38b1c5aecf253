"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments on the host
(no kernel is launched by any test in this file)."""
import ctypes
import os
import re

import pytest

import paper_2306_07629_amd as sq
from paper_2306_07629_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 1 << 20   # a fake, 16-byte aligned, never dereferenced device address


def header_symbols():
    text = open(os.path.join(ROOT, "include", "sqllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sqllm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sq.lib()
    names = header_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names
    for n in names:                                   # the Python binding offers the same names
        if n not in ("sqllm_last_error_string", "sqllm_status_string"):
            assert hasattr(sq, n) or hasattr(binding, n), n
    assert sq.sqllm_version() >= 100


def expect(status_name, fn, *args):
    with pytest.raises(sq.SqllmError) as e:
        fn(*args, stream=0)
    assert binding.STATUS_NAMES[e.value.status] == status_name, str(e.value)
    assert len(str(e.value)) > len(status_name) + 2          # carries a message


def test_lut_gemv_argument_errors():
    f = sq.sqllm_lut_gemv
    expect("SQLLM_ERR_BITS", f, 4, 128, 1, 1, A, A, A, A)
    expect("SQLLM_ERR_BITS", f, 4, 128, 5, 1, A, A, A, A)
    expect("SQLLM_ERR_SHAPE", f, -1, 128, 3, 1, A, A, A, A)
    expect("SQLLM_ERR_SHAPE", f, 4, 0, 3, 1, A, A, A, A)
    expect("SQLLM_ERR_SHAPE", f, 4, 100, 3, 1, A, A, A, A)
    expect("SQLLM_ERR_SHAPE", f, 4, 64, 4, 1, A, A, A, A)
    expect("SQLLM_ERR_SHAPE", f, 4, 28672 + 128, 3, 1, A, A, A, A)
    expect("SQLLM_ERR_BATCH", f, 4, 128, 3, 0, A, A, A, A)
    expect("SQLLM_ERR_BATCH", f, 4, 128, 3, 17, A, A, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 3, 1, None, A, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 3, 1, A, None, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 3, 1, A, A, None, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 3, 1, A, A, A, None)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 3, 1, A + 4, A, A, A)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 3, 1, A, A + 8, A, A)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 3, 1, A, A, A + 2, A)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 3, 1, A, A, A, A + 1)


def test_sparse_argument_errors():
    f = sq.sqllm_csr_spmv
    expect("SQLLM_ERR_NNZ", f, 4, 128, -1, 1, A, A, A, A, A)
    expect("SQLLM_ERR_NNZ", f, 4, 128, 1 << 31, 1, A, A, A, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 5, 1, None, A, A, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 5, 1, A, None, A, A, A)
    expect("SQLLM_ERR_NULL", f, 4, 128, 5, 1, A, A, None, A, A)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 5, 1, A + 2, A, A, A, A)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 5, 1, A, A, A + 1, A, A)
    expect("SQLLM_ERR_SHAPE", f, 4, 130, 5, 1, A, A, A, A, A)
    g = sq.sqllm_dense_sparse_matvec
    expect("SQLLM_ERR_NULL", g, 4, 128, 3, 5, 1, A, A, None, A, A, A, A)
    expect("SQLLM_ERR_BITS", g, 4, 128, 8, 5, 1, A, A, A, A, A, A, A)
    expect("SQLLM_ERR_NNZ", g, 4, 128, 3, -2, 1, A, A, A, A, A, A, A)
    expect("SQLLM_ERR_BATCH", g, 4, 128, 3, 0, 100, A, A, None, None, None, A, A)
    h = sq.sqllm_csr_spmv_rowwise
    expect("SQLLM_ERR_NNZ", h, 4, 128, -1, 1, A, A, A, A, A)


def test_multi_layer_argument_errors():
    ok = (4, 128, 3, 5, A, A, A, A, A, A, A)
    f = lambda layers: sq.sqllm_dense_sparse_matvec_multi(layers, stream=0)
    with pytest.raises(sq.SqllmError) as e:
        f([ok, (4, 100, 3, 5, A, A, A, A, A, A, A)])
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_SHAPE" and "layer 1" in str(e.value)
    with pytest.raises(sq.SqllmError) as e:
        f([ok, ok, (4, 128, 4, 5, A, A, A, A, A, A, A)])
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_BITS" and "layer 2" in str(e.value)
    with pytest.raises(sq.SqllmError) as e:
        f([(4, 128, 3, 5, A, A, None, A, A, A, A)])
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_NULL" and "layer 0" in str(e.value)
    with pytest.raises(sq.SqllmError) as e:
        f([(4, 128, 3, 0, A, A, None, None, None, A + 2, A)])
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_ALIGN"
    L = sq.lib()
    assert L.sqllm_dense_sparse_matvec_multi(-1, None, None) == binding.STATUS_NAMES.index("SQLLM_ERR_SHAPE")
    assert L.sqllm_dense_sparse_matvec_multi(3, None, None) == binding.STATUS_NAMES.index("SQLLM_ERR_NULL")
    assert L.sqllm_dense_sparse_matvec_multi(0, None, None) == 0
    f([(0, 128, 3, 0, A, A, None, None, None, A, A)] * 3)          # only empty layers: nothing is enqueued, no HIP call


def test_plan_argument_errors_and_sizes():
    n = sq.sqllm_csr_plan_bytes(4096, 4096, 75497)
    assert n % 256 == 0 and 75497 * 4 < n < 75497 * 24     # slots 15 % above the mean plus a worst-case overflow region
    assert sq.sqllm_csr_plan_bytes(8, 128, 0) % 256 == 0 and sq.sqllm_csr_plan_bytes(0, 128, 0) >= 0
    assert sq.sqllm_csr_plan_bytes(22016, 8192, 811598) > sq.sqllm_csr_plan_bytes(11008, 8192, 405799)
    for bad in ((4, 100, 5), (-1, 128, 5), (4, 128, -1)):
        with pytest.raises(sq.SqllmError):
            sq.sqllm_csr_plan_bytes(*bad)
    f = sq.sqllm_csr_plan_build
    nb = sq.sqllm_csr_plan_bytes(4, 128, 5)
    expect("SQLLM_ERR_NULL", f, 4, 128, 5, A, A, A, None, nb)
    expect("SQLLM_ERR_NULL", f, 4, 128, 5, None, A, A, A, nb)
    expect("SQLLM_ERR_ALIGN", f, 4, 128, 5, A, A, A, A + 128, nb)
    expect("SQLLM_ERR_SHAPE", f, 4, 128, 5, A, A, A, A, nb - 256)
    expect("SQLLM_ERR_SHAPE", f, 4, 130, 5, A, A, A, A, nb)
    expect("SQLLM_ERR_NNZ", f, 4, 128, -5, A, A, A, A, nb)
    f(0, 128, 0, A, None, None, A, 4096, stream=0)                   # nothing to do, nothing enqueued
    # with a plan the CSR arrays of a one-column call may be NULL; the plan must be aligned
    g = lambda plan: sq.sqllm_dense_sparse_matvec(0, 128, 3, 5, 1, A, A, None, None, None, A, A, stream=0, plan=plan)
    g(A)
    with pytest.raises(sq.SqllmError) as e:
        sq.sqllm_dense_sparse_matvec(4, 128, 3, 5, 1, A, A, None, None, None, A, A, stream=0, plan=A + 64)
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_ALIGN"
    with pytest.raises(sq.SqllmError) as e:                          # B = 2 ignores the plan and needs the CSR arrays
        sq.sqllm_dense_sparse_matvec(4, 128, 3, 5, 2, A, A, None, None, None, A, A, stream=0, plan=A)
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_NULL"


def test_debug_and_baseline_argument_errors():
    expect("SQLLM_ERR_NULL", sq.sqllm_unpack_indices, 4, 128, 3, A, None)
    expect("SQLLM_ERR_BITS", sq.sqllm_unpack_indices, 4, 128, 1, A, A)
    expect("SQLLM_ERR_NULL", sq.sqllm_dequantize, 4, 128, 4, A, A, None)
    expect("SQLLM_ERR_ALIGN", sq.sqllm_dequantize, 4, 128, 4, A, A, A + 1)
    expect("SQLLM_ERR_SHAPE", sq.sqllm_fp16_gemv, 4, 12, 1, A, A, A)
    expect("SQLLM_ERR_NULL", sq.sqllm_fp16_gemv, 4, 16, 1, None, A, A)
    expect("SQLLM_ERR_ALIGN", sq.sqllm_fp16_gemv, 4, 16, 1, A + 2, A, A)
    expect("SQLLM_ERR_BATCH", sq.sqllm_fp16_gemv, 4, 16, 0, A, A, A)


def test_empty_problem_is_ok_without_a_device():
    # M == 0: nothing to do, nothing is enqueued, no HIP call is made
    sq.sqllm_lut_gemv(0, 128, 3, 1, A, A, A, A, stream=0)
    sq.sqllm_dense_sparse_matvec(0, 128, 4, 0, 1, A, A, None, None, None, A, A, stream=0)
    sq.sqllm_csr_spmv(0, 128, 0, 1, None, None, None, A, A, stream=0)
    sq.sqllm_unpack_indices(0, 128, 3, A, A, stream=0)


def test_algorithmic_bytes_and_status_strings():
    assert sq.sqllm_algorithmic_bytes(11008, 4096, 3, 202899, 1) == 18376054
    assert sq.sqllm_algorithmic_bytes(4096, 4096, 4, 75497, 1) == 9005434
    assert sq.sqllm_algorithmic_bytes(4096, 4096, 4, 0, 1) == 4096 * 4096 // 2 + 4096 * 32 + 2 * 8192
    L = sq.lib()
    assert L.sqllm_status_string(0) == b"SQLLM_OK" and L.sqllm_status_string(3) == b"SQLLM_ERR_SHAPE"


def test_quantize_argument_errors():
    f = sq.sqllm_quantize_layer
    ws = sq.sqllm_quantize_workspace_bytes(4, 128)
    assert ws > 0 and ws % 4 == 0
    ok = dict(M=4, N=128, bits=3, max_iter=8, w=A, sens=A, n_lo=1, n_hi=1, n_sens=1, workspace=A, workspace_bytes=ws,
              qidx=A, lut=A, rowptr=A, cols=A, vals=A)

    def call(status, **over):
        a = dict(ok, **over)
        expect(status, lambda stream: f(a["M"], a["N"], a["bits"], a["max_iter"], a["w"], a["sens"], a["n_lo"], a["n_hi"], a["n_sens"],
                                        a["workspace"], a["workspace_bytes"], a["qidx"], a["lut"], a["rowptr"], a["cols"], a["vals"], None, stream))

    call("SQLLM_ERR_BITS", bits=1)
    call("SQLLM_ERR_BITS", bits=5)
    call("SQLLM_ERR_SHAPE", N=100)
    call("SQLLM_ERR_SHAPE", M=-1)
    call("SQLLM_ERR_SHAPE", M=1 << 20, N=4096)                 # 2^32 weights: beyond the histogram counters
    call("SQLLM_ERR_SHAPE", max_iter=-1)
    call("SQLLM_ERR_SHAPE", workspace_bytes=ws - 4)
    call("SQLLM_ERR_NNZ", n_lo=4 * 128)
    call("SQLLM_ERR_NNZ", n_hi=-1)
    call("SQLLM_ERR_NNZ", n_sens=4 * 128)
    for name in ("w", "sens", "workspace", "qidx", "lut", "rowptr", "cols", "vals"):
        call("SQLLM_ERR_NULL", **{name: None})
    call("SQLLM_ERR_ALIGN", w=A + 8)
    call("SQLLM_ERR_ALIGN", sens=A + 2)
    call("SQLLM_ERR_ALIGN", lut=A + 4)
    call("SQLLM_ERR_ALIGN", rowptr=A + 2)
    call("SQLLM_ERR_ALIGN", vals=A + 1)
    # nothing to extract: cols / vals may be NULL; M == 0: nothing is enqueued
    f(0, 128, 3, 8, A, A, 0, 0, 0, A, ws, A, A, A, None, None, None, 0)
    assert sq.sqllm_extraction_counts(4096, 4096, 0.004, 0.0005) == (33554, 33554, 8388)
    assert sq.sqllm_extraction_counts(4096, 4096, 0.0, 0.0) == (0, 0, 0)
    assert sq.sqllm_extraction_counts(11008, 4096, 0.004, 0.0005) == (int(0.004 * 11008 * 4096 / 2),) * 2 + (int(0.0005 * 11008 * 4096),)
    for bad in ((-1, 128, 0.1, 0.1), (4, 128, -0.1, 0.0), (4, 128, 0.6, 0.5)):
        with pytest.raises(sq.SqllmError):
            sq.sqllm_extraction_counts(*bad)
