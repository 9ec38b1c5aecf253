"""Seeded random small layers through every one-column path -- sparse term from the CSR arrays, from a plan, and several layers in
one launch with four and with eight rows per workgroup -- against the CPU oracle and against each other.  The shapes are drawn to
hit what fixed lists miss: row counts around multiples of 4 and 8, a last workgroup of one to seven rows, rows without nonzeros,
nonzero shares from none to a third of the matrix, widths from one 128-column group to several waves with a ragged last slice."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3


def draw(rng):
    M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 17, 31, 33, 40, 63, 70]))
    N = int(rng.choice([128, 256, 384, 1024, 2048, 2176, 4096, 4224, 6144, 8192, 11008]))
    bits = int(rng.choice([2, 3, 4]))
    frac = float(rng.choice([0.0, 0.001, 0.0045, 0.02, 0.3]))
    skew = [None, (0.1, 0.5), (0.01, 0.3)][int(rng.integers(0, 3))]
    if frac > 0.0045:
        skew = None                                              # a heavy row cannot hold more nonzeros than it has columns
    return M, N, bits, frac, skew


def check(L, y, what):
    y_ref, absdot = oracle.layer_matvec(L)
    err = np.abs(y.cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
    assert (err <= TOL * absdot + 2.0 ** -25).all(), (what, L.M, L.N, L.bits, L.nnz, float(np.max(err / (TOL * absdot + 2.0 ** -25))))


@pytest.mark.parametrize("seed", range(40))
def test_random_layers_through_all_one_column_paths(seed):
    import torch
    import paper_2306_07629_amd as sq
    rng = np.random.default_rng(31000 + seed)
    bits = int(rng.choice([2, 3, 4]))
    specs = []
    for _ in range(5):
        M, N, _b, frac, skew = draw(rng)
        specs.append((M, N, frac, skew))
    print(f"random shapes seed={seed} bits={bits} specs={specs}", flush=True)
    layers = [gen.make_layer(M, N, bits, frac=frac, skew=skew, seed=32000 + 10 * seed + k) for k, (M, N, frac, skew) in enumerate(specs)]
    csr = [sq.DeviceLayer(L) for L in layers]
    planned = [sq.DeviceLayer(L).build_plan() for L in layers]
    y_csr, y_plan = [], []
    for L, D, P in zip(layers, csr, planned):
        y_csr.append(D.matvec().clone()); check(L, y_csr[-1], "CSR arrays")
        y_plan.append(P.matvec().clone()); check(L, y_plan[-1], "plan")
        # the dense term does not depend on where the sparse term comes from
        assert torch.equal(D.lut_gemv().clone(), P.lut_gemv())
    # one launch per class, four rows per workgroup (all layers are narrower than 16384 columns)
    for group, want in ((csr, y_csr), (planned, y_plan)):
        for D in group:
            D.y.fill_(0x7BFF)
        sq.sqllm_dense_sparse_matvec_multi([D.descriptor() for D in group])
        torch.cuda.synchronize()
        for D, y1 in zip(group, want):
            assert torch.equal(D.y, y1)
    # a 16384-wide planned layer in front makes the planned launch take eight rows per workgroup: same bits
    wide = gen.make_layer(int(rng.choice([3, 8, 13])), 16384, bits, frac=0.0045, skew=None, seed=33000 + seed)
    W = sq.DeviceLayer(wide).build_plan()
    yw = W.matvec().clone(); check(wide, yw, "plan, wide")
    for D in planned + [W]:
        D.y.fill_(0x7BFF)
    sq.sqllm_dense_sparse_matvec_multi([W.descriptor()] + [D.descriptor() for D in planned])
    torch.cuda.synchronize()
    assert torch.equal(W.y, yw)
    for D, y1 in zip(planned, y_plan):
        assert torch.equal(D.y, y1)
