"""Pins of the quantiser oracle (oracle/quant_oracle.py) against things other than itself: exact rational
arithmetic, a library k-means, brute force on tiny inputs, closed forms and the inequalities the paper's Sec. 4.1-4.2
rest on.  No GPU."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import gen
from oracle import quant_oracle as qo


def f16(vals):
    return np.asarray(vals, dtype=np.float16).view(np.uint16)


def exact(bits):
    return [Fraction(float(v)) for v in np.asarray(bits, dtype=np.uint16).view(np.float16)]


# ------------------------------------------------------------------------------------------------ number formats
def test_half_to_fixed_is_exact_for_every_finite_pattern():
    bits = np.array([b for b in range(65536) if (b >> 10) & 31 != 31], dtype=np.uint16)
    fixed = qo.half_to_fixed(bits)
    vals = bits.view(np.float16).astype(np.float64)           # fp16 -> fp64 is exact
    assert np.array_equal(fixed.astype(np.float64), vals * 2.0 ** 24)
    assert np.all(np.abs(fixed) < 2 ** 41)


def test_half_key_orders_like_the_reals():
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 65536, 4000).astype(np.uint16)
    bits = bits[((bits >> 10) & 31) != 31]
    vals = bits.view(np.float16).astype(np.float64)
    keys = qo.half_key(bits).astype(np.int64)
    order = np.argsort(keys, kind="stable")
    assert np.all(np.diff(vals[order]) >= 0)
    a, b = f16([-0.0]), f16([0.0])
    assert qo.half_key(a)[0] < qo.half_key(b)[0]


def test_exact_integer_to_double_matches_python_rounding():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        hi = int(rng.integers(-2 ** 40, 2 ** 40))
        lo = int(rng.integers(0, 2 ** 47))
        assert float(qo._exact_to_f64(hi, lo)) == float(hi * 2 ** 32 + lo)     # Python: correctly rounded int -> float


# ------------------------------------------------------------------------------------------------ the split (Sec. 4.2)
def test_thresholds_on_a_hand_example():
    # 12 weights -5 .. 6 (distinct), sensitivities 1 .. 12 in another order
    w = f16([[3, -5, 0, 6, -1, 2], [5, -4, 1, -3, 4, -2]])
    s = np.array([[1, 2, 3, 4, 5, 12], [6, 7, 11, 8, 9, 10]], dtype=np.uint16)
    thr = qo.thresholds(w, s, 2, 1, 2)
    key_min, key_max, s_thr = thr
    assert key_min == qo.half_key(f16([-3]))[0] and key_max == qo.half_key(f16([5]))[0] and s_thr == 10
    mask = qo.split_mask(w, s, thr)
    # extracted: w < -3 -> {-5, -4};  w > 5 -> {6};  s > 10 -> {12, 11}
    assert mask.tolist() == [[False, True, False, True, False, True], [False, True, True, False, False, False]]
    rowptr, cols, vals = qo.csr_from_mask(w, mask)
    assert rowptr.tolist() == [0, 3, 5] and cols.tolist() == [1, 3, 5, 1, 2]
    assert vals.tolist() == f16([-5, 6, 2, -4, 1]).tolist()


def test_split_is_the_papers_decomposition():
    """W = D + S, S = W[w < T_min or w > T_max] plus the most sensitive weights; counts hit the targets when
    there are no ties at the thresholds, and never exceed them."""
    M, N = 64, 512
    w = gen.make_weights(M, N, 11)
    s = gen.make_sens(M, N, 11)
    total = M * N
    n_lo = n_hi = int(0.002 * total)
    n_sens = int(0.0005 * total)
    thr = qo.thresholds(w, s, n_lo, n_hi, n_sens)
    mask = qo.split_mask(w, s, thr)
    vals = w.view(np.float16).astype(np.float64)
    t_min = np.sort(vals.ravel())[n_lo]
    t_max = np.sort(vals.ravel())[total - 1 - n_hi]
    low, high, sen = vals < t_min, vals > t_max, s > np.sort(s.ravel())[total - 1 - n_sens]
    assert np.array_equal(mask, low | high | sen)
    assert low.sum() <= n_lo and high.sum() <= n_hi and sen.sum() <= n_sens
    rowptr, cols, v = qo.csr_from_mask(w, mask)
    assert rowptr[-1] == mask.sum() and np.all(np.diff(rowptr) >= 0)
    dense = np.where(mask, 0, w)
    sparse = np.zeros_like(w)
    for i in range(M):
        c = cols[rowptr[i]:rowptr[i + 1]]
        assert np.all(np.diff(c) > 0)
        sparse[i, c] = v[rowptr[i]:rowptr[i + 1]]
    assert np.array_equal(np.where(mask, sparse, dense), w)
    # range contraction (Sec. 4.2: removing a fraction of a percent of the weights shrinks the range several-fold)
    assert (vals.max() - vals.min()) > 2.0 * (vals[~mask].max() - vals[~mask].min())


def test_zero_counts_extract_nothing():
    w = gen.make_weights(8, 128, 3)
    s = gen.make_sens(8, 128, 3)
    assert not qo.split_mask(w, s, qo.thresholds(w, s, 0, 0, 0)).any()


# ------------------------------------------------------------------------------------------------ Lloyd (Sec. 4.1)
def rational_objective(wq, sq, centroids, assign):
    return sum(Fraction(int(si)) * (wi - centroids[ai]) ** 2 for wi, si, ai in zip(wq, sq, assign))


def test_converged_state_is_a_fixed_point_in_exact_arithmetic():
    N, K = 1024, 8
    w = gen.make_weights(1, N, 21)[0]
    s = np.maximum(gen.make_sens(1, N, 21)[0], 1)
    dense = np.ones(N, dtype=bool)
    c, it, a = qo.kmeans_row(w, s, dense, K, 200)
    assert 0 < it < 200
    wq = exact(w)
    cq = [Fraction(float(v)) for v in c]
    assert all(cq[k] <= cq[k + 1] for k in range(K - 1))
    # every weight sits with a nearest centroid (up to the fp32 rounding of the mid-point sum)
    for wi, ai in zip(wq, a):
        best = min(abs(wi - ck) for ck in cq)
        assert abs(wi - cq[ai]) - best <= Fraction(1, 2 ** 30)
    # every centroid is the sensitivity-weighted mean of its members, rounded to fp32 (double rounding: <= 1 ulp)
    for k in range(K):
        members = [j for j in range(N) if a[j] == k]
        assert members
        mean = sum(Fraction(int(s[j])) * wq[j] for j in members) / sum(int(s[j]) for j in members)
        assert abs(cq[k] - mean) <= abs(mean) * Fraction(1, 2 ** 23)


def test_objective_never_increases():
    N, K = 512, 8
    w = gen.make_weights(1, N, 22)[0]
    s = np.maximum(gen.make_sens(1, N, 22)[0], 1)
    dense = np.ones(N, dtype=bool)
    wq = exact(w)
    prev = None
    for iters in range(0, 12):
        c, it, a = qo.kmeans_row(w, s, dense, K, iters)
        obj = rational_objective(wq, s, [Fraction(float(v)) for v in c], a)
        if prev is not None:
            assert obj <= prev * (1 + Fraction(1, 10 ** 6))
        prev = obj
        if it < iters:
            break


def test_agrees_with_a_library_kmeans():
    sklearn_cluster = pytest.importorskip("sklearn.cluster")
    N, K = 2048, 8
    w = gen.make_weights(1, N, 23)[0]
    s = np.maximum(gen.make_sens(1, N, 23)[0], 1)
    dense = np.ones(N, dtype=bool)
    c, it, a = qo.kmeans_row(w, s, dense, K, 300)
    wf = w.view(np.float16).astype(np.float64)
    init = np.sort(wf)[[((2 * k + 1) * N) // (2 * K) for k in range(K)]].reshape(-1, 1)     # equal-count start
    km = sklearn_cluster.KMeans(n_clusters=K, init=init, n_init=1, max_iter=300, tol=0.0, algorithm="lloyd")
    km.fit(wf.reshape(-1, 1), sample_weight=s.astype(np.float64))
    centers = km.cluster_centers_.ravel()
    assert np.all(np.diff(centers) > 0)
    np.testing.assert_allclose(c.astype(np.float64), centers, rtol=2e-6, atol=1e-9)
    assert (km.labels_ != a).mean() < 2e-3          # weights on a cluster boundary may fall either way


def test_brute_force_on_tiny_rows():
    """Optimal 1-D clusters are contiguous in sorted order: enumerate every split."""
    rng = np.random.default_rng(5)
    for trial in range(6):
        n, K = 9, 4
        w = f16(np.sort(rng.normal(0, 0.05, n)))
        s = rng.integers(1, 50, n).astype(np.uint16)
        wq = exact(w)
        best = None
        for cuts in itertools.combinations(range(1, n), K - 1):
            bounds = (0,) + cuts + (n,)
            obj = Fraction(0)
            for g in range(K):
                js = range(bounds[g], bounds[g + 1])
                mean = sum(Fraction(int(s[j])) * wq[j] for j in js) / sum(int(s[j]) for j in js)
                obj += sum(Fraction(int(s[j])) * (wq[j] - mean) ** 2 for j in js)
            best = obj if best is None or obj < best else best
        c, it, a = qo.kmeans_row(w, s, np.ones(n, dtype=bool), K, 100)
        got = rational_objective(wq, s, [Fraction(float(v)) for v in c], a)
        assert got >= best * (1 - Fraction(1, 10 ** 6))
    # three tight, well separated groups and three centroids: Lloyd reaches the optimum (each group its mean)
    w = f16([-1.0, -0.99, -1.01, 0.0, 0.01, -0.01, 1.0, 1.01, 0.99])
    s = np.ones(9, dtype=np.uint16)
    c, it, a = qo.kmeans_row(w, s, np.ones(9, dtype=bool), 4, 100)
    assert len(set(a[[0, 1, 2]])) == 1 and len(set(a[[3, 4, 5]])) <= 2 and len(set(a[[6, 7, 8]])) <= 2
    for k in set(a.tolist()):
        members = [exact(w)[j] for j in range(9) if a[j] == k]
        mean = sum(members) / len(members)
        assert abs(Fraction(float(c[k])) - mean) <= Fraction(1, 2 ** 22)


def test_degenerate_rows():
    K = 8
    w = f16([0.25] * 64)
    s = np.ones(64, dtype=np.uint16)
    c, it, a = qo.kmeans_row(w, s, np.ones(64, dtype=bool), K, 10)
    assert np.all(c == np.float32(0.25)) and np.all(a == 0)
    c, it, a = qo.kmeans_row(w, s, np.zeros(64, dtype=bool), K, 10)          # nothing dense
    assert np.all(c == 0) and it == 0 and a.size == 0
    # members without sensitivity do not move their centroid
    w = f16([0.0, 1.0, 2.0, 3.0])
    s = np.array([1, 0, 0, 1], dtype=np.uint16)
    c, it, a = qo.kmeans_row(w, s, np.ones(4, dtype=bool), 4, 10)
    assert c.tolist() == [0.0, 1.0, 2.0, 3.0] and a.tolist() == [0, 1, 2, 3]


def test_final_indices_and_tables():
    lut = f16([-0.5, -0.1, 0.05, 0.6])
    w = f16([-0.3, -0.31, 0.0, -0.025, 0.325, 0.33, 5.0, -7.0])
    dense = np.array([1, 1, 1, 1, 1, 1, 0, 0], dtype=bool)
    idx = qo.final_indices(w, dense, lut)
    # -0.3 is nearer to -0.1 (fp16 values: |-0.3+0.1| < |-0.3+0.5|);  extracted entries take the entry nearest to 0
    wq, cq = exact(w), exact(lut)
    for j in range(6):
        d = [abs(wq[j] - ck) for ck in cq]
        assert idx[j] == d.index(min(d))
    assert idx[6] == 2 and idx[7] == 2
    # an exact tie goes to the lower index
    lut2 = f16([-1.0, 1.0, 2.0, 4.0])
    assert qo.final_indices(f16([0.0, 1.5, 3.0]), np.ones(3, dtype=bool), lut2).tolist() == [0, 1, 2]


def test_the_inequalities_the_method_rests_on():
    """Sec. 4.1: non-uniform (k-means) tables represent a heavy-tailed row better than a uniform grid, under the
    plain error (Eq. 1) and under the sensitivity-weighted error (Eq. 4); and the weighted iteration, started from
    the unweighted solution's tables, does not make the weighted error worse."""
    M, N, bits = 6, 2048, 3
    K = 1 << bits
    w = gen.make_weights(M, N, 31)
    s = np.maximum(gen.make_sens(M, N, 31), 1)
    ones = np.ones(N, dtype=np.uint16)
    dense = np.ones(N, dtype=bool)
    for i in range(M):
        c_w, _, _ = qo.kmeans_row(w[i], s[i], dense, K, 100)
        c_u, _, _ = qo.kmeans_row(w[i], ones, dense, K, 100)
        lut_w, lut_u = qo.float_to_half_bits(c_w), qo.float_to_half_bits(c_u)
        wf = w[i].view(np.float16).astype(np.float64)
        grid = f16(np.linspace(wf.min(), wf.max(), K))                       # round-to-nearest uniform quantiser
        obj = lambda lut, sv: qo.objective(w[i], sv, dense, lut, qo.final_indices(w[i], dense, lut))
        assert obj(lut_u, ones) < obj(grid, ones)
        assert obj(lut_w, s[i]) < obj(grid, s[i])
        ranks = [((2 * k + 1) * N) // (2 * K) for k in range(K)]
        lut_0 = qo.float_to_half_bits(np.sort(w[i].view(np.float16).astype(np.float32))[ranks])   # the equal-count start
        assert obj(lut_w, s[i]) <= obj(lut_0, s[i])


def test_quantize_layer_round_trip_feeds_the_matvec_oracle():
    """The quantiser's output is a valid layer for the matvec: W_eff = lut[idx] (+ extracted values) stays close to W."""
    import oracle
    M, N, bits = 16, 256, 4
    w = gen.make_weights(M, N, 41)
    s = gen.make_sens(M, N, 41)
    total = M * N
    q = qo.quantize_layer(w, s, bits, int(0.002 * total), int(0.002 * total), int(0.0005 * total), max_iter=50)
    assert np.all(np.diff(q["lut"].view(np.float16).astype(np.float64), axis=1) >= 0)
    L = gen.hand_layer(q["idx"], q["lut"].view(np.float16), bits, q["rowptr"], q["cols"], q["vals"].view(np.float16),
                       gen.make_x(N, 1, 41).view(np.float16))
    y, absdot = oracle.layer_matvec(L)
    y16, _ = oracle.fp16_matvec(w, L.x)
    # the dense part of W_eff is within half a table step of W; compare the products loosely
    err = np.abs(y - y16).max()
    assert err < 0.25 * np.abs(y16).max() + 0.05
    # extracted positions: the table entry nearest to zero plus the full value
    mask = q["mask"]
    lutv = q["lut"].view(np.float16).astype(np.float64)
    for i in range(M):
        z = np.argmin(np.abs(lutv[i]))
        assert np.all(q["idx"][i][mask[i]] == z)
