"""Host-side check that the kernels never read past the end of an input array.

The kernels avoid divergent bounds checks: tail lanes, tail rows and surplus sparse batches load CLAMPED addresses whose
results are neutralised later.  A GPU test cannot show that such a load stays inside its array (an over-read of a few bytes
lands in mapped memory of the allocator's pool and the result is still right), so this test re-computes, from the clamping
formulas the kernels use (`j0c`, `min(r0 + u, M - 1)`, `min(p, P1 - 1)`, `last_t`, the slots of the activation windows), every
address range they touch, for every shape of the GPU test lists, and asserts that it lies inside the array."""
import numpy as np
import pytest

SLICE, LANE_ELEMS, WAVE = 2048, 32, 64

SHAPES = [  # (M, N, bits, B) -- the shapes of the GPU parity lists, ragged ones first
    (1, 128, 2, 1), (5, 2176, 3, 1), (3, 128, 4, 1), (2, 28672, 3, 1), (37, 128, 3, 1), (301, 2176, 4, 1), (67, 11008, 3, 1),
    (33, 22016, 2, 1), (4097, 4096, 3, 1), (9, 28672, 4, 1), (11008, 4096, 3, 1), (8192, 22016, 3, 1),
    (5, 2176, 3, 16), (19, 128, 4, 5), (33, 256, 2, 8), (17, 384, 3, 3), (65, 2304, 3, 5), (8200, 256, 3, 16), (8209, 128, 4, 11),
    (9, 28672, 3, 16), (40, 28672, 2, 9), (70, 2304, 4, 2), (65, 8192, 2, 4), (130, 4096, 4, 12),
]


def rowptr_for(M, N, seed):
    """a skewed CSR pattern: empty rows, a full row, a ragged tail"""
    rng = np.random.default_rng(seed)
    counts = rng.integers(0, 6, size=M)
    counts[rng.integers(0, M)] = min(N, 700)
    if M > 3:
        counts[M - 1] = 0
    return np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)


def one_column_kernel_reads(M, N, bits, rowptr, R):
    """yields (array name, first byte, one past the last byte) for every load of the one-column kernel"""
    W = (N + SLICE - 1) // SLICE
    K = 1 << bits
    row_bytes = 2 * K
    unit = min(row_bytes, 16)
    lpr = row_bytes // unit
    lanes = np.arange(WAVE)
    for r0 in sorted({0, ((M - 1) // R) * R, ((M // 2) // R) * R}):
        nrows = min(R, M - r0)
        for w in range(W):
            j0 = w * SLICE + lanes * LANE_ELEMS
            j0c = np.where(j0 < N, j0, N - LANE_ELEMS)
            yield "x", int((2 * j0c).min()), int((2 * j0c + 64).max())
            for u in range(R):
                row = min(r0 + u, M - 1)
                off = row * (N * bits // 8) + (j0c // 32) * bits * 4
                yield "qidx", int(off.min()), int((off + 4 * bits).max())
        fetch = lanes[lanes < R * lpr]
        row = np.minimum(r0 + fetch // lpr, M - 1)
        off = row * row_bytes + (fetch % lpr) * unit
        yield "lut", int(off.min()), int((off + unit).max())
        rp = [int(rowptr[r0 + min(k, nrows)]) for k in range(R + 1)]
        yield "rowptr", 4 * r0, 4 * (r0 + nrows) + 4
        P0, P1 = rp[0], rp[R]
        nbatch = (P1 - P0 + WAVE - 1) // WAVE
        if nbatch > 0:
            NW, UB = W + 1, 8  # dense waves and the sparse wave
            for b0 in range(0, nbatch + NW * UB, 1):             # every batch slot a round can touch, surplus ones included
                p = np.minimum(P0 + b0 * WAVE + lanes, P1 - 1)
                assert (p >= P0).all()
                yield "cols", int(4 * p.min()), int(4 * p.max() + 4)
                yield "vals", int(2 * p.min()), int(2 * p.max() + 2)


def sixteen_column_kernel_reads(M, N, bits, B, rowptr):
    RG = 2 if M >= 8192 else 1
    R = 16 * RG
    nwin = N // 128
    NW = min(nwin, 8)
    K = 1 << bits
    lanes = np.arange(WAVE)
    r, q = lanes % 16, lanes // 16
    nnz = int(rowptr[-1])
    if B in (4, 8, 12, 16):
        B4 = B // 4
    elif B == 2:
        B4 = 5
    else:
        B4 = 0
    BT = 2 if B4 == 5 else 4 * B4
    for r0 in sorted({0, ((M - 1) // R) * R}):
        raw_lanes = R * (2 * K) // min(2 * K, 16)
        unit = min(2 * K, 16)
        tid = np.arange(raw_lanes)
        row = np.minimum(r0 + tid * unit // (2 * K), M - 1)
        off = row * 2 * K + (tid * unit) % (2 * K)
        yield "lut", int(off.min()), int((off + unit).max())
        for rg in range(RG):
            lo = np.minimum(r0 + 16 * rg + r, M)
            yield "rowptr", int(4 * lo.min()), int(4 * np.minimum(lo + 1, M).max() + 4)
        for wave in range(NW):
            last_t = wave + ((nwin - 1 - wave) // NW) * NW
            for t in sorted({wave, min(wave + NW, last_t), min(wave + 2 * NW, last_t), last_t}):
                for rg in range(RG):
                    row = np.minimum(r0 + 16 * rg + r, M - 1)
                    off = (row * (N * bits // 32) + (4 * t + q) * bits) * 4
                    yield "qidx", int(off.min()), int((off + 4 * bits).max())
                wbase = t * 128 * B * 2                            # byte offset of the window in x[N][B]
                if B4 in (2, 4):
                    for i in range(B4):
                        off = wbase + (64 * i + lanes) * 16
                        yield "x", int(off.min()), int(off.max() + 16)
                elif B4 > 0:
                    off = wbase + lanes * 4 * BT
                    yield "x", int(off.min()), int(off.max() + max(8, 4 * BT))
                else:
                    qd = 16 * B
                    for qq in range(4):
                        for ii in range(4):
                            off = wbase + 4 * qq * qd + 4 * np.minimum(64 * ii + lanes, qd - 1)
                            yield "x", int(off.min()), int(off.max() + 4)
        if nnz > 0:
            e4 = 4 * (lanes // 16) + (lanes % 4)
            for sj in (0, int(rowptr[min(r0 + R, M)]) // 16, (nnz - 1) // 16):
                pl = np.minimum(16 * sj + e4, nnz - 1)
                assert (pl >= 0).all()
                yield "cols", int(4 * pl.min()), int(4 * pl.max() + 4)
                yield "vals", int(2 * pl.min()), int(2 * pl.max() + 2)


def plan_sections(M, N, nnz):
    """sizes in bytes of the five sections of a plan (the layout documented with PlanLayout in csrc/sqllm_kernels.h): blocks of four
    rows whatever the rows per workgroup of the kernel"""
    W = (N + SLICE - 1) // SLICE
    n_q = (M + 3) // 4
    groups = nnz // 16 + M // 2 + 1
    C = max(1, min(W, (groups * 115 // 100 + 4 * n_q - 1) // (4 * n_q)))
    ov_cap = (nnz // 16 + M) // 4 + n_q + 1
    return W, n_q, C, ov_cap, {"slot_entries": n_q * C * 256, "slot_tags": n_q * C * 4, "ov_desc": n_q * 8, "ov_entries": ov_cap * 256, "ov_tags": ov_cap * 4}


def planned_kernel_reads(M, N, rowptr, R):
    """every load the planned one-column kernel with R rows per workgroup issues into the plan: per block of four rows the slot batch
    of each wave, the overflow descriptor, the overflow batches requested ahead (clamped into the overflow sections whatever the
    descriptor holds) and those of the loop"""
    nnz = int(rowptr[-1])
    W, n_q, C, ov_cap, size = plan_sections(M, N, nnz)
    counts = np.diff(rowptr)
    groups = np.add.reduceat((np.concatenate([counts, np.zeros(n_q * 4 - M, dtype=counts.dtype)]) + 15) // 16, np.arange(0, n_q * 4, 4))
    ov_nb = (np.maximum(groups - 4 * C, 0) + 3) // 4
    ov_first = np.concatenate([[0], np.cumsum(ov_nb)[:-1]])
    assert int(ov_first[-1] + ov_nb[-1]) <= ov_cap                # the capacity bound the layout promises
    Q = R // 4
    UP, UO = (2 if Q == 1 else 1), 8
    n_wg = (M + R - 1) // R
    heavy = int(np.argmax(ov_nb)) // Q
    for block in sorted({0, n_wg - 1, n_wg // 2, heavy}):
        for wave in range(W):
            for q in range(Q):
                quad = min(block * Q + q, n_q - 1)
                sb = quad * C + min(wave, C - 1)
                yield "slot_entries", sb * 256, sb * 256 + 256
                yield "slot_tags", sb * 4, sb * 4 + 4
                yield "ov_desc", 8 * quad, 8 * quad + 8
                first, nb = int(ov_first[quad]), (int(ov_nb[quad]) if block * Q + q < n_q else 0)
                for k in range(UP):
                    b = min(first + min(wave + k * W, max(nb - 1, 0)), ov_cap - 1)
                    assert b >= 0
                    yield "ov_entries", b * 256, b * 256 + 256
                    yield "ov_tags", b * 4, b * 4 + 4
                ob = wave + UP * W
                while ob < nb:
                    for k in range(UO):
                        b = first + min(ob + k * W, nb - 1)
                        yield "ov_entries", b * 256, b * 256 + 256
                        yield "ov_tags", b * 4, b * 4 + 4
                    ob += UO * W


@pytest.mark.parametrize("M,N,bits,B", [s for s in SHAPES if s[3] == 1])
def test_every_load_of_the_planned_kernel_stays_inside_its_section(M, N, bits, B):
    rowptr = rowptr_for(M, N, M + N + bits)
    size = plan_sections(M, N, int(rowptr[-1]))[4]
    reads = list(planned_kernel_reads(M, N, rowptr, 4)) + list(planned_kernel_reads(M, N, rowptr, 8))   # either may be launched
    assert len(reads) > 4
    for name, lo, hi in reads:
        assert 0 <= lo and hi <= size[name], (name, lo, hi, size[name])


def test_plan_sections_add_up_to_the_size_the_library_reports():
    import paper_2306_07629_amd as sq
    for M, N, bits, B in SHAPES:
        nnz = int(rowptr_for(M, N, M + N + bits)[-1])
        size = plan_sections(M, N, nnz)[4]
        assert sum((v + 255) & ~255 for v in size.values()) == sq.sqllm_csr_plan_bytes(M, N, nnz)


@pytest.mark.parametrize("M,N,bits,B", SHAPES)
def test_every_load_stays_inside_its_array(M, N, bits, B):
    rowptr = rowptr_for(M, N, M + N + bits)
    nnz = int(rowptr[-1])
    size = {"x": 2 * N * B, "qidx": M * N * bits // 8, "lut": M * 2 * (1 << bits), "rowptr": 4 * (M + 1), "cols": 4 * nnz, "vals": 2 * nnz}
    if B == 1:
        # rows per workgroup as the launcher picks them
        R = 8 if (N + SLICE - 1) // SLICE >= 8 else 4
        reads = list(one_column_kernel_reads(M, N, bits, rowptr, R)) + list(one_column_kernel_reads(M, N, bits, rowptr, 12 - R))
    else:
        reads = list(sixteen_column_kernel_reads(M, N, bits, B, rowptr))
    assert len(reads) > 4
    for name, lo, hi in reads:
        assert 0 <= lo and hi <= size[name], (name, lo, hi, size[name])
