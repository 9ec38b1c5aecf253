"""The plan of the sparse term (sqllm_csr_plan_build) and the one-column kernel that reads it: the re-layout is checked entry by
entry against the CSR arrays (integer work: bit-exact), the planned matvec against the CPU oracle to the same bars as the
unplanned one, on small ragged layers, degenerate sparsity patterns (overflow of heavy rows) and the full benchmark shapes."""
import numpy as np
import pytest

import gen
import oracle

pytestmark = pytest.mark.gpu
TOL = 2e-3
SEED = 20230613


def layout(M, N, nnz):
    """the offsets of the plan's sections, as documented with PlanLayout in csrc/sqllm_kernels.h"""
    W = (N + 2047) // 2048
    R = 4                                                          # rows per block of the plan, whatever the kernel's rows per workgroup
    n_wg = (M + R - 1) // R
    groups = nnz // 16 + M // 2 + 1
    C = max(1, min(W, (groups * 115 // 100 + 4 * n_wg - 1) // (4 * n_wg)))
    ov_cap = (nnz // 16 + M) // 4 + n_wg + 1
    up = lambda v: (v + 255) & ~255
    off, o = {}, 0
    for name, size in (("slot_entries", n_wg * C * 256), ("slot_tags", n_wg * C * 4), ("ov_desc", n_wg * 8), ("ov_entries", ov_cap * 256), ("ov_tags", ov_cap * 4)):
        off[name] = o
        o += up(size)
    return R, n_wg, C, ov_cap, off, o


def decode_plan(buf, L):
    """(row, col, fp16 bits) of every valid entry of the plan, workgroup by workgroup, in storage order"""
    import paper_2306_07629_amd as sq
    R, n_wg, C, ov_cap, off, total = layout(L.M, L.N, L.nnz)
    assert total == sq.sqllm_csr_plan_bytes(L.M, L.N, L.nnz) == buf.size
    se = buf[off["slot_entries"]:off["slot_entries"] + n_wg * C * 256].view(np.uint32).reshape(n_wg, C, 64)
    st = buf[off["slot_tags"]:off["slot_tags"] + n_wg * C * 4].reshape(n_wg, C, 4)
    od = buf[off["ov_desc"]:off["ov_desc"] + n_wg * 8].view(np.int32).reshape(n_wg, 2)
    oe = buf[off["ov_entries"]:off["ov_entries"] + ov_cap * 256].view(np.uint32).reshape(ov_cap, 64)
    ot = buf[off["ov_tags"]:off["ov_tags"] + ov_cap * 4].reshape(ov_cap, 4)
    out = []
    assert od[0, 0] == 0 and (np.diff(od[:, 0]) == od[:-1, 1]).all() and od[-1, 0] + od[-1, 1] <= ov_cap
    for b in range(n_wg):
        batches = [(se[b, k], st[b, k]) for k in range(C)] + [(oe[od[b, 0] + k], ot[od[b, 0] + k]) for k in range(od[b, 1])]
        seen_invalid = False
        for ent, tags in batches:
            for gi in range(4):
                t = int(tags[gi])
                if not t & 0x80:
                    seen_invalid = True
                    assert (ent[16 * gi:16 * gi + 16] == 0).all()
                    continue
                assert not seen_invalid, "a valid group after an empty one"
                row, cnt = b * R + (t & 7), ((t >> 3) & 15) + 1
                e = ent[16 * gi:16 * gi + cnt]
                assert (ent[16 * gi + cnt:16 * gi + 16] == 0).all()
                out.extend((row, int(v & 0x7FFF), int(v >> 16)) for v in e)
                assert ((e >> 15) & 1 == 0).all()
    return out


CASES = [  # (M, N, bits, frac, skew)
    (37, 128, 3, 0.02, None), (301, 2176, 4, 0.0045, (0.1, 0.5)), (130, 4096, 3, 0.0045, None), (67, 11008, 3, 0.0045, (0.1, 0.5)),
    (33, 22016, 3, 0.0045, (0.01, 0.3)), (9, 28672, 2, 0.0045, None), (1, 128, 3, 0.05, None), (5, 16384, 4, 0.01, None), (1030, 4096, 2, 0.001, (0.1, 0.5)),
]


@pytest.mark.parametrize("M,N,bits,frac,skew", CASES)
def test_plan_holds_exactly_the_csr_entries_and_the_planned_matvec_matches_the_oracle(M, N, bits, frac, skew):
    import paper_2306_07629_amd as sq
    print(f"plan case M={M} N={N} bits={bits} frac={frac} skew={skew}", flush=True)
    L = gen.make_layer(M, N, bits, frac=frac, skew=skew, seed=8000 + M + N + bits)
    D = sq.DeviceLayer(L).build_plan()
    got = decode_plan(D.plan.cpu().numpy(), L)
    rows = np.repeat(np.arange(M), np.diff(L.rowptr))
    want = list(zip(rows.tolist(), L.cols.tolist(), L.vals.tolist()))
    assert got == want                                            # same entries, same (row-major, column-ascending) order
    y_ref, absdot = oracle.layer_matvec(L)
    y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
    err = np.abs(y - y_ref)
    assert (err <= TOL * absdot + 2.0 ** -25).all(), float(np.max(err / (TOL * absdot + 2.0 ** -25)))
    tight = 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -24 + (N + 64) * 2.0 ** -24 * absdot
    assert (err <= tight).all()
    # without the plan: the same entry point on the CSR arrays, same tolerance, results equal up to the order of additions
    D2 = sq.DeviceLayer(L)
    y2 = D2.matvec().cpu().numpy().view(np.float16).astype(np.float64)
    assert (np.abs(y - y2) <= 2.0 ** -10 * np.abs(y2) + 2.0 ** -24).all()
    # run to run
    a = D.matvec().cpu().numpy().copy()
    for _ in range(3):
        assert np.array_equal(D.matvec().cpu().numpy(), a)


def test_heavy_rows_overflow_the_slots():
    """one row holds every column, its neighbour thousands, the rest of the matrix next to nothing: most batches of that
    workgroup live in the overflow region and are shared by all waves"""
    import paper_2306_07629_amd as sq
    M, N, bits = 64, 8192, 3
    rng = np.random.default_rng(8)
    idx = rng.integers(0, 8, size=(M, N), dtype=np.uint8)
    lut = np.sort((rng.standard_normal((M, 8)) * 0.05).astype(np.float16), axis=1)
    counts = np.zeros(M, dtype=np.int64); counts[17] = N; counts[18] = 5000; counts[19] = 17; counts[40] = 16; counts[41] = 1; counts[63] = 33
    rowptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    cols = np.concatenate([np.sort(rng.choice(N, c, replace=False)) for c in counts if c]).astype(np.int32)
    vals = (rng.standard_normal(cols.size) * 0.1).astype(np.float16)
    x = rng.standard_normal((N, 1)).astype(np.float16)
    L = gen.hand_layer(idx, lut, bits, rowptr, cols, vals, x)
    D = sq.DeviceLayer(L).build_plan()
    got = decode_plan(D.plan.cpu().numpy(), L)
    rows = np.repeat(np.arange(M), np.diff(L.rowptr))
    assert got == list(zip(rows.tolist(), L.cols.tolist(), L.vals.tolist()))
    y_ref, a_ref = oracle.layer_matvec(L)
    y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
    assert (np.abs(y - y_ref) <= TOL * a_ref).all()


@pytest.mark.parametrize("M,N,skew", [(8192, 8192, (0.01, 0.30)), (22016, 8192, (0.01, 0.30)), (8192, 22016, (0.01, 0.30)), (11008, 4096, (0.10, 0.50)),
                                      (4096, 11008, (0.10, 0.50)), (13824, 5120, None)])
def test_planned_matvec_at_the_benchmark_shapes(M, N, skew):
    import paper_2306_07629_amd as sq
    print(f"planned full size {M}x{N}", flush=True)
    L = gen.make_layer(M, N, 3, frac=0.0045, skew=skew, seed=gen.layer_seed(SEED, 9, M // 100 + N // 1000))
    D = sq.DeviceLayer(L).build_plan()
    y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
    y_ref, absdot = oracle.layer_matvec(L)
    err = np.abs(y - y_ref)
    assert np.isfinite(y).all() and (err <= TOL * absdot).all(), float(np.max(err / (TOL * absdot)))
    assert (err <= 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -24 + (N + 4096) * 2.0 ** -24 * absdot).all()


def test_planned_layers_stacked_and_in_one_launch_give_the_bits_of_separate_calls():
    """q, k, v stacked into one 3 M x N layer, and the three layers in one multi-layer launch: with a plan every row's nonzeros
    are summed in an order of their own, so even the fused result is bit for bit that of the separate calls"""
    import torch
    import paper_2306_07629_amd as sq
    from test_gpu_stacked_and_unit import stack
    layers = [gen.make_layer(1024, 4096, 3, frac=0.0045, skew=(0.10, 0.50), seed=gen.layer_seed(SEED, 10, k)) for k in range(3)]
    for L in layers[1:]:
        L.x = layers[0].x
    devs = [sq.DeviceLayer(L).build_plan() for L in layers]
    sep = [D.matvec().clone() for D in devs]
    S = stack(layers)
    DS = sq.DeviceLayer(S).build_plan()
    ys = DS.matvec()
    assert torch.equal(ys, torch.cat(sep))
    for D in devs:
        D.y.zero_()
    sq.sqllm_dense_sparse_matvec_multi([D.descriptor() for D in devs])
    torch.cuda.synchronize()
    for D, y1 in zip(devs, sep):
        assert torch.equal(D.y, y1)


def planned_multi_equals_separate(specs, bits, seed0):
    import torch
    import paper_2306_07629_amd as sq
    layers = [gen.make_layer(M, N, bits, frac=frac, skew=skew, seed=seed0 + k) for k, (M, N, frac, skew) in enumerate(specs)]
    devs = [sq.DeviceLayer(L).build_plan() for L in layers]
    sep = []
    for D in devs:
        sep.append(D.matvec().clone())                              # four rows per workgroup for rows below 16384 columns
        D.y.fill_(0x7BFF)
    torch.cuda.synchronize()
    sq.sqllm_dense_sparse_matvec_multi([D.descriptor() for D in devs])
    torch.cuda.synchronize()
    for k, (L, D, y1) in enumerate(zip(layers, devs, sep)):
        assert torch.equal(D.y, y1), f"layer {k} ({L.M}x{L.N}) differs from the separate call"
        y_ref, absdot = oracle.layer_matvec(L)
        err = np.abs(D.y.cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
        assert (err <= TOL * absdot + 2.0 ** -25).all(), f"layer {k}"


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_planned_multi_launch_with_eight_rows_per_workgroup_gives_the_bits_of_the_four_row_launches(bits):
    """A 16384-wide layer makes the whole planned launch run with eight rows per workgroup, i.e. two plan blocks per workgroup;
    the narrow layers' own launches use four.  Row counts that leave the last workgroup one block, or a block of one to three rows;
    layers without nonzeros (no plan: they go to a launch of their own class); heavy rows that overflow the slot."""
    specs = [(33, 16384, 0.0045, None), (37, 128, 0.02, None), (301, 2176, 0.0045, (0.1, 0.5)), (4, 4096, 0.01, None), (12, 8192, 0.0045, None),
             (64, 128, 0.0, None), (203, 1024, 0.0045, (0.01, 0.3)), (1, 128, 0.05, None), (70, 11008, 0.0045, (0.1, 0.5)), (5, 2048, 0.3, None)]
    print(f"planned multi, eight rows, {bits}-bit", flush=True)
    planned_multi_equals_separate(specs, bits, 8800 + bits)


def test_planned_multi_launch_of_many_workgroups_switches_to_eight_rows_and_keeps_the_bits():
    """three 11008x4096 and two 4096x4096 layers: more than 4096 eight-row workgroups, so the launch takes eight rows per
    workgroup where the single-layer launches take four"""
    specs = [(11008, 4096, 0.0045, (0.1, 0.5))] * 3 + [(4096, 4096, 0.0045, (0.1, 0.5))] * 2
    print("planned multi, full size", flush=True)
    planned_multi_equals_separate(specs, 3, 8900)


def test_four_full_size_decoder_blocks_in_one_call():
    """28 full-size layers of a 7B-shaped model (four decoder blocks, a seed per layer) in ONE multi-layer call, eight rows per
    workgroup; every y against the oracle and against the layer's own launch"""
    block = [(4096, 4096, 0.0045, (0.1, 0.5))] * 4 + [(11008, 4096, 0.0045, (0.1, 0.5))] * 2 + [(4096, 11008, 0.0045, (0.1, 0.5))]
    print("planned multi, four decoder blocks", flush=True)
    planned_multi_equals_separate(block * 4, 3, 9000)


@pytest.mark.parametrize("bits", [2, 4])
def test_forty_small_planned_layers_split_into_launches_of_sixteen(bits):
    """more planned layers than one launch holds (16): launches of 16, 16 and 8 layers, four rows per workgroup"""
    rng = np.random.default_rng(91 + bits)
    specs = [(int(rng.integers(1, 40)), int(rng.choice([128, 256, 1024, 2176, 4096])), float(rng.choice([0.0045, 0.02])), None) for _ in range(40)]
    print(f"planned multi, forty layers, {bits}-bit", flush=True)
    planned_multi_equals_separate(specs, bits, 9100 + bits)


def test_three_hundred_mixed_layers_in_one_call_are_regrouped_and_keep_the_bits():
    """300 small layers in one call, with and without a plan, widths of 1 to 11 waves in shuffled order: the call sorts them into
    groups (plan or none, waves per workgroup, row class) and launches group by group; every y must be that of the layer's own
    call, and rows the call does not own stay untouched"""
    import torch
    import paper_2306_07629_amd as sq
    rng = np.random.default_rng(4242)
    widths = [128, 2048, 2176, 4096, 6144, 8192, 11008, 16384, 22016]
    layers, devs = [], []
    for k in range(300):
        M, N = int(rng.integers(1, 20)), int(rng.choice(widths))
        frac = float(rng.choice([0.0, 0.0045, 0.03]))
        L = gen.make_layer(M, N, 3, frac=frac, skew=None, seed=9300 + k)
        D = sq.DeviceLayer(L)
        if rng.integers(0, 2) and L.nnz > 0:
            D.build_plan()
        layers.append(L)
        devs.append(D)
    print("mixed multi, 300 layers", flush=True)
    sep = []
    for D in devs:
        sep.append(D.matvec().clone())
        D.y.fill_(0x7BFF)
    torch.cuda.synchronize()
    sq.sqllm_dense_sparse_matvec_multi([D.descriptor() for D in devs])
    torch.cuda.synchronize()
    for k, (L, D, y1) in enumerate(zip(layers, devs, sep)):
        assert torch.equal(D.y, y1), f"layer {k} ({L.M}x{L.N}, nnz {L.nnz}) differs from the separate call"
    y_ref, absdot = oracle.layer_matvec(layers[7])
    err = np.abs(devs[7].y.cpu().numpy().view(np.float16).astype(np.float64) - y_ref)
    assert (err <= TOL * absdot + 2.0 ** -25).all()
