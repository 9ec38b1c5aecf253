"""GPU tests of how the library sits in a HIP program: graph capture and replay, non-default streams,
guard regions around every output buffer, repeated calls."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _f64(t):
    return t.cpu().numpy().view(np.float16).astype(np.float64)


@pytest.mark.parametrize("B", [1, 16, 7])
def test_graph_replays_match_the_eager_result(B):
    """the benchmark replays a captured graph: every replay must give the eager result (no memset nodes, no
    host-side state baked into the capture); one column, and the matrix-core kernel with both activation paths"""
    import torch
    import paper_2306_07629_amd as sq
    L = gen.make_layer(1030, 4096, 3, frac=0.0045, skew=(0.1, 0.5), B=B, seed=31)
    D = sq.DeviceLayer(L)
    eager = D.matvec().clone()
    torch.cuda.synchronize()
    y_ref, absdot = oracle.layer_matvec(L)
    assert (np.abs(_f64(eager) - y_ref) <= TOL * absdot).all()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            D.matvec()
            D.lut_gemv(accumulate=1)          # second node depends on the first through y
    torch.cuda.synchronize()
    D.lut_gemv()                               # eager reference of the two-node sequence: y = fp16(fused) + dense
    want = None
    for rep in range(4):
        D.y.fill_(12345)                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = D.y.clone()
        if want is None:
            D.matvec(); D.lut_gemv(accumulate=1); torch.cuda.synchronize()
            want = D.y.clone()
        assert torch.equal(got, want), f"replay {rep}"


def test_graph_replays_of_planned_and_multi_layer_calls_match_the_eager_result():
    """what the decode-step benchmark replays: a planned single-layer call (plan built before the capture) and a multi-layer
    call, whose descriptors are copied into the kernel arguments at capture time (the host array is dropped before the first
    replay)"""
    import torch
    import paper_2306_07629_amd as sq
    layers = [gen.make_layer(M, N, 3, frac=0.0045, skew=(0.1, 0.5), seed=60 + k) for k, (M, N) in enumerate([(1030, 4096), (517, 11008), (33, 16384)])]
    devs = [sq.DeviceLayer(L).build_plan() for L in layers]
    eager = [D.matvec().clone() for D in devs]
    torch.cuda.synchronize()
    for L, y in zip(layers, eager):
        y_ref, absdot = oracle.layer_matvec(L)
        assert (np.abs(_f64(y) - y_ref) <= TOL * absdot).all()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            devs[0].matvec()                                                       # planned, one layer
            desc = sq.layer_descriptors([D.descriptor() for D in devs[1:]])
            sq.sqllm_dense_sparse_matvec_multi(desc)                               # planned, two layers, eight rows per workgroup
    del desc
    torch.cuda.synchronize()
    for rep in range(4):
        for D in devs:
            D.y.fill_(12345)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (D, y) in enumerate(zip(devs, eager)):
            assert torch.equal(D.y, y), f"replay {rep}, layer {k}"


def test_non_default_stream_and_back_to_back_calls():
    import torch
    import paper_2306_07629_amd as sq
    L = gen.make_layer(515, 2304, 4, frac=0.0045, seed=32)
    D = sq.DeviceLayer(L)
    base = D.matvec().clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for _ in range(50):
            D.matvec(stream=s)
    s.synchronize()
    assert torch.equal(D.y, base)


@pytest.mark.parametrize("bits,M,N,B", [(3, 37, 2176, 1), (4, 70, 4096, 2), (3, 9, 11008, 4), (3, 40, 2176, 16), (4, 33, 384, 7), (2, 50, 1024, 12)])
def test_guard_regions_around_outputs_stay_untouched(bits, M, N, B):
    """y, idx_out and w_out are carved out of larger buffers filled with a sentinel"""
    import torch
    import paper_2306_07629_amd as sq
    L = gen.make_layer(M, N, bits, frac=0.0045, skew=(0.1, 0.5), B=B, seed=40 + M)
    D = sq.DeviceLayer(L)
    pad = 4096
    SENT = 0x5A5A

    def carve(nelem, dtype, sent):
        buf = torch.full((nelem + 2 * pad,), sent, dtype=dtype, device="cuda")
        return buf, buf[pad:pad + nelem]

    ybuf, y = carve(M * B, torch.int16, SENT)
    D.y = y.view(M, B)
    D.matvec(); D.lut_gemv(); D.csr_spmv(accumulate=1); D.csr_spmv(rowwise=True)
    torch.cuda.synchronize()
    assert bool((ybuf[:pad] == SENT).all()) and bool((ybuf[pad + M * B:] == SENT).all())
    ibuf, idx = carve(M * N, torch.uint8, 0xA5)
    sq.sqllm_unpack_indices(M, N, bits, D.qidx, idx)
    wbuf, w = carve(M * N, torch.int16, SENT)
    sq.sqllm_dequantize(M, N, bits, D.qidx, D.lut, w)
    torch.cuda.synchronize()
    assert bool((ibuf[:pad] == 0xA5).all()) and bool((ibuf[pad + M * N:] == 0xA5).all())
    assert bool((wbuf[:pad] == SENT).all()) and bool((wbuf[pad + M * N:] == SENT).all())
    assert np.array_equal(idx.view(M, N).cpu().numpy(), oracle.unpack(M, N, bits, L.qidx))
    assert np.array_equal(w.view(M, N).cpu().numpy().view(np.uint16), oracle.dequant(M, N, bits, L.qidx, L.lut))
