"""Several independent layers in one launch (sqllm_dense_sparse_matvec_multi): every y is bit for bit the y of a separate
sqllm_dense_sparse_matvec call and within the tolerance of the CPU oracle."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3


def run(specs, bits, seed0):
    import torch
    import paper_2306_07629_amd as sq
    layers = [gen.make_layer(M, N, bits, frac=frac, skew=skew, seed=seed0 + k) for k, (M, N, frac, skew) in enumerate(specs)]
    devs = [sq.DeviceLayer(L) for L in layers]
    separate = []
    for D in devs:
        separate.append(D.matvec().clone())
        D.y.fill_(0x7BFF)                                           # a value no result has: every row must be rewritten
    torch.cuda.synchronize()
    sq.sqllm_dense_sparse_matvec_multi([D.descriptor() for D in devs])
    torch.cuda.synchronize()
    for k, (L, D, y1) in enumerate(zip(layers, devs, separate)):
        assert torch.equal(D.y, y1), f"layer {k} ({L.M}x{L.N}) differs from the separate call"
        y_ref, absdot = oracle.layer_matvec(L)
        err = np.abs(D.y.cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
        assert (err <= TOL * absdot + 2.0 ** -25).all(), f"layer {k}"


def test_one_decoder_block_in_one_launch():
    """seven layers with the shape mix of a decoder block (scaled-down row counts, full widths): 2 and 6 waves per workgroup
    in one launch, ragged last workgroups, row skew"""
    specs = [(515, 4096, 0.0045, (0.1, 0.5))] * 4 + [(1377, 4096, 0.0045, (0.1, 0.5))] * 2 + [(513, 11008, 0.0045, (0.1, 0.5))]
    print("multi: decoder-block mix", flush=True)
    run(specs, 3, 7000)


@pytest.mark.parametrize("bits", [2, 4])
def test_more_layers_than_one_launch_holds_and_both_row_classes(bits):
    """eleven layers; a 16384-wide layer in the middle forces a launch boundary of its own (8 rows per workgroup); layers without
    nonzeros and with a single row"""
    specs = [(70, 2048, 0.0045, None), (1, 128, 0.0, None), (300, 2176, 0.01, (0.1, 0.5)), (33, 16384, 0.0045, None), (64, 128, 0.0, None),
             (9, 22016, 0.0045, None), (129, 4096, 0.0005, None), (37, 128, 0.02, None), (200, 1024, 0.0045, (0.01, 0.3)), (5, 8192, 0.0045, None),
             (77, 2304, 0.0045, None)]
    print(f"multi: eleven layers, {bits}-bit", flush=True)
    run(specs, bits, 7100 + bits)


def test_full_size_block_of_the_7b_step():
    specs = [(4096, 4096, 0.0045, (0.1, 0.5))] * 2 + [(11008, 4096, 0.0045, (0.1, 0.5)), (4096, 11008, 0.0045, (0.1, 0.5))]
    print("multi: full-size 7B layers", flush=True)
    run(specs, 3, 7200)


def test_more_layers_than_one_launch_holds():
    """forty small layers: the call splits them into launches of at most SQLLM_MAX_LAYERS_PER_LAUNCH (16)"""
    rng = np.random.default_rng(77)
    specs = [(int(rng.integers(1, 40)), int(rng.choice([128, 256, 1024, 2176, 4096])), float(rng.choice([0.0, 0.0045, 0.02])), None) for _ in range(40)]
    print("multi: forty layers", flush=True)
    run(specs, 3, 7300)

