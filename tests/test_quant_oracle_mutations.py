"""The pins of the quantiser oracle must notice plausible mistakes.  Each case plants ONE mistake in a copy of the
oracle's Python source (on the CPU, never in the GPU path), loads it as a module of its own and checks that at
least one pin of a small battery fails; the untouched source passes the same battery."""
import itertools
import os
import types
from fractions import Fraction

import numpy as np
import pytest

import gen
from oracle import quant_oracle as qo_good

SRC = os.path.join(os.path.dirname(qo_good.__file__), "quant_oracle.py")

MUTATIONS = {
    "negative keys not inverted": ("return np.where(neg, ~b, b | 0x8000).astype(np.uint16)", "return np.where(neg, b, b | 0x8000).astype(np.uint16)"),
    "fixed point loses the implicit one": ("mag = np.where(e == 0, m, (m + 1024) << np.maximum(e - 1, 0))", "mag = np.where(e == 0, m, m << np.maximum(e - 1, 0))"),
    "fixed point exponent off by one": ("(m + 1024) << np.maximum(e - 1, 0)", "(m + 1024) << np.maximum(e, 0)"),
    "lower threshold one rank off": ("return int(keys[n_lo]),", "return int(keys[max(n_lo - 1, 0)]),"),
    "upper threshold from the wrong end": ("int(keys[total - 1 - n_hi])", "int(keys[n_hi])"),
    "ties at the threshold extracted": ("return (k < key_min) | (k > key_max) | (sens > s_thr)", "return (k <= key_min) | (k > key_max) | (sens > s_thr)"),
    "sensitive weights not extracted": ("return (k < key_min) | (k > key_max) | (sens > s_thr)", "return (k < key_min) | (k > key_max)"),
    "CSR values taken from the wrong place": ("w_bits[rows, cols].astype(np.uint16)", "w_bits[rows, cols - 1].astype(np.uint16)"),
    "row pointers not accumulated": ("rowptr[1:] = np.cumsum(counts)", "rowptr[1:] = counts"),
    "start ranks without the half step": ("order[((2 * k + 1) * n) // (2 * K)]", "order[(k * n) // K]"),
    "assignment ties to the upper index": ("a = (t[None, :] < two_w[:, None]).sum(axis=1)", "a = (t[None, :] <= two_w[:, None]).sum(axis=1)"),
    "assignment against the centroids instead of the mid-points": ("t = (c[:-1] + c[1:]).astype(np.float32)", "t = (c[:-1] + c[:-1]).astype(np.float32)"),
    "unweighted mean": ("s0 = int(s[m].sum())", "s0 = int(m.sum())"),
    "weights squared in the mean": ("p = s * wfix ", "p = s * s * wfix "),
    "high word dropped": ("s1 = _exact_to_f64(int(p_hi[m].sum()), int(p_lo[m].sum()))", "s1 = _exact_to_f64(0, int(p_lo[m].sum()))"),
    "fixed point scale": ("np.float64(2.0 ** -24)", "np.float64(2.0 ** -23)"),
    "stops after the first update": ("        it += 1\n", "        it += 1\n        break\n"),
    "empty cluster zeroed": ("            if s0 > 0:\n", "            if s0 == 0:\n                c[k] = 0\n            if s0 > 0:\n"),
    "final ties to the upper index": ("idx = (t[None, :] < (2 * wfix)[:, None]).sum(axis=1)", "idx = (t[None, :] <= (2 * wfix)[:, None]).sum(axis=1)"),
    "extracted positions get index 0": ("return np.where(dense, idx, zero).astype(np.uint8)", "return np.where(dense, idx, 0).astype(np.uint8)"),
    "entry nearest to zero by signed value": ("zero = int(np.argmin(np.abs(cfix)))", "zero = int(np.argmin(cfix))"),
    "tables from the extracted weights too": ("        dense = ~mask[i]\n", "        dense = np.ones_like(mask[i])\n"),
}


def load(source: str) -> types.ModuleType:
    mod = types.ModuleType("quant_oracle_under_test")
    exec(compile(source, "quant_oracle_under_test.py", "exec"), mod.__dict__)
    return mod


def f16(vals):
    return np.asarray(vals, dtype=np.float16).view(np.uint16)


def exact(bits):
    return [Fraction(float(v)) for v in np.asarray(bits, dtype=np.uint16).view(np.float16)]


def battery(qo):
    """a fast subset of the pins in test_quant_oracle_pins.py; raises AssertionError on the first mismatch"""
    # number formats
    bits = np.array([0x0001, 0x03FF, 0x0400, 0x3C00, 0xBC00, 0x7BFF, 0x8001, 0x2E66, 0xAE66], dtype=np.uint16)
    assert np.array_equal(qo.half_to_fixed(bits).astype(np.float64), bits.view(np.float16).astype(np.float64) * 2.0 ** 24)
    vals = bits.view(np.float16).astype(np.float64)
    assert np.all(np.diff(vals[np.argsort(qo.half_key(bits).astype(np.int64))]) >= 0)
    # the hand example of the split
    w = f16([[3, -5, 0, 6, -1, 2], [5, -4, 1, -3, 4, -2]])
    s = np.array([[1, 2, 3, 4, 5, 12], [6, 7, 11, 8, 9, 10]], dtype=np.uint16)
    thr = qo.thresholds(w, s, 2, 1, 2)
    mask = qo.split_mask(w, s, thr)
    assert mask.tolist() == [[False, True, False, True, False, True], [False, True, True, False, False, False]]
    rowptr, cols, v = qo.csr_from_mask(w, mask)
    assert rowptr.tolist() == [0, 3, 5] and cols.tolist() == [1, 3, 5, 1, 2] and v.tolist() == f16([-5, 6, 2, -4, 1]).tolist()
    # ties at a threshold stay dense
    wt = f16([[1, 1, 1, 2, 3, 3, 3, 3]])
    st = np.ones((1, 8), dtype=np.uint16)
    assert qo.split_mask(wt, st, qo.thresholds(wt, st, 1, 1, 0)).sum() == 0
    # Lloyd: fixed point in exact arithmetic, sensitivity-weighted means
    N, K = 512, 8
    wr = gen.make_weights(1, N, 21)[0]
    sr = np.maximum(gen.make_sens(1, N, 21)[0], 1)
    dense = np.ones(N, dtype=bool)
    c, it, a = qo.kmeans_row(wr, sr, dense, K, 200)
    assert 1 < it < 200
    wq, cq = exact(wr), [Fraction(float(x)) for x in c]
    for wi, ai in zip(wq, a):
        assert abs(wi - cq[ai]) - min(abs(wi - ck) for ck in cq) <= Fraction(1, 2 ** 30)
    for k in range(K):
        members = [j for j in range(N) if a[j] == k]
        assert members
        mean = sum(Fraction(int(sr[j])) * wq[j] for j in members) / sum(int(sr[j]) for j in members)
        assert abs(cq[k] - mean) <= abs(mean) * Fraction(1, 2 ** 23)
    # the start is the equal-count one: with no update allowed the centroids are order statistics
    c0, it0, _ = qo.kmeans_row(wr, sr, dense, K, 0)
    assert it0 == 0
    srt = np.sort(wr.view(np.float16).astype(np.float32))
    assert c0.tolist() == [float(srt[((2 * k + 1) * N) // (2 * K)]) for k in range(K)]
    # an assignment tie goes to the lower centroid; a member without sensitivity does not move its centroid
    c, it, a = qo.kmeans_row(f16([0.0, 1.0, 2.0, 3.0]), np.array([1, 0, 0, 1], dtype=np.uint16), np.ones(4, dtype=bool), 4, 10)
    assert c.tolist() == [0.0, 1.0, 2.0, 3.0] and a.tolist() == [0, 1, 2, 3]
    c, it, a = qo.kmeans_row(f16([0.0, 1.0, 2.0]), np.ones(3, dtype=np.uint16), np.ones(3, dtype=bool), 2, 0)
    assert c.tolist() == [0.0, 2.0] and a.tolist() == [0, 0, 1]
    # brute force on a tiny row
    rng = np.random.default_rng(5)
    n, K2 = 9, 3
    wb = f16(np.sort(rng.normal(0, 0.05, n)))
    sb = rng.integers(1, 50, n).astype(np.uint16)
    wbq = exact(wb)
    best = None
    for cuts in itertools.combinations(range(1, n), K2 - 1):
        bounds = (0,) + cuts + (n,)
        obj = Fraction(0)
        for g in range(K2):
            js = range(bounds[g], bounds[g + 1])
            mean = sum(Fraction(int(sb[j])) * wbq[j] for j in js) / sum(int(sb[j]) for j in js)
            obj += sum(Fraction(int(sb[j])) * (wbq[j] - mean) ** 2 for j in js)
        best = obj if best is None or obj < best else best
    c, it, a = qo.kmeans_row(wb, sb, np.ones(n, dtype=bool), 4, 100)
    got = sum(Fraction(int(si)) * (wi - Fraction(float(c[ai]))) ** 2 for wi, si, ai in zip(wbq, sb, a))
    assert got <= best            # four centroids can only do better than the best three
    # final indices and the whole pass
    lut = f16([-0.5, -0.1, 0.05, 0.6])
    wf = f16([-0.3, -0.31, 0.0, -0.025, 0.325, 0.33, 5.0, -7.0])
    dn = np.array([1, 1, 1, 1, 1, 1, 0, 0], dtype=bool)
    idx = qo.final_indices(wf, dn, lut)
    wfq, lq = exact(wf), exact(lut)
    for j in range(6):
        d = [abs(wfq[j] - ck) for ck in lq]
        assert idx[j] == d.index(min(d))
    assert idx[6] == 2 and idx[7] == 2
    assert qo.final_indices(f16([0.0, 1.5, 3.0]), np.ones(3, dtype=bool), f16([-1.0, 1.0, 2.0, 4.0])).tolist() == [0, 1, 2]
    M2, N2 = 8, 256
    w2, s2 = gen.make_weights(M2, N2, 41), gen.make_sens(M2, N2, 41)
    q = qo.quantize_layer(w2, s2, 3, 4, 4, 2, max_iter=50)
    wv = w2.view(np.float16).astype(np.float64)
    lutv = q["lut"].view(np.float16).astype(np.float64)
    for i in range(M2):
        dense_i = ~q["mask"][i]
        # no table entry lies outside the range of the row's dense weights (outliers do not pull the tables)
        assert lutv[i].min() >= wv[i][dense_i].min() - 1e-3 and lutv[i].max() <= wv[i][dense_i].max() + 1e-3
        assert np.all(q["idx"][i][q["mask"][i]] == np.argmin(np.abs(lutv[i])))
    assert q["iters"].min() >= 2


def test_the_untouched_oracle_passes_the_battery():
    battery(load(open(SRC).read()))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_a_planted_mistake_is_noticed(name):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation anchor not found: {old!r}"
    mutant = load(src.replace(old, new, 1))
    with pytest.raises(Exception):
        battery(mutant)
