"""Pins for the filtered-sampling checker (min-p, top-k, top-p in that order): with both filters
off it is the plain rule; degenerate settings are greedy; closed forms on a few tokens; the kept
set is nested; and a brute-force restatement on tiny vocabularies agrees."""
import itertools

import numpy as np
import pytest


def _one(oracle, x, T, top_p, u, top_k=0, min_p=0.0):
    x = np.asarray([x], dtype=np.float32)
    r = oracle.sample_tokens_filtered(x, np.float32([T]), np.float32([top_p]), np.float32([u]),
                                      np.int32([top_k]), np.float32([min_p]))
    return int(r["token"][0]), int(r["kept"][0])


def test_filters_off_is_the_plain_rule(oracle):
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((40, 777)) * 3).astype(np.float32)
    T = rng.choice([0.0, 0.3, 0.8, 1.0], 40).astype(np.float32)
    tp = rng.choice([0.1, 0.7, 0.95, 1.0], 40).astype(np.float32)
    u = rng.random(40, dtype=np.float32)
    a = oracle.sample_tokens(x, T, tp, u)
    for tk, mp in ((None, None), (np.zeros(40, np.int32), np.zeros(40, np.float32)),
                   (np.full(40, 777, np.int32), None), (np.full(40, 5000, np.int32), np.zeros(40, np.float32))):
        b = oracle.sample_tokens_filtered(x, T, tp, u, tk, mp)
        assert np.array_equal(a["token"], b["token"]) and np.array_equal(a["kept"], b["kept"])
        assert np.allclose(a["cdf_lo"], b["cdf_lo"], rtol=0, atol=1e-15)


def test_top_k_one_and_min_p_one_are_greedy(oracle):
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((30, 300)) * 2).astype(np.float32)
    u = rng.random(30, dtype=np.float32)
    T = np.full(30, 0.9, np.float32)
    one = np.ones(30, np.float32)
    arg = x.argmax(axis=1)
    a = oracle.sample_tokens_filtered(x, T, one, u, np.ones(30, np.int32), None)
    b = oracle.sample_tokens_filtered(x, T, one, u, None, one)
    assert np.array_equal(a["token"], arg) and np.array_equal(b["token"], arg)
    assert np.all(a["kept"] == 1) and np.all(b["kept"] == 1)


def test_closed_forms_on_four_tokens(oracle):
    # logits ln 8, ln 4, ln 2, ln 1 at T = 1: p (relative to the maximum) = 1, 1/2, 1/4, 1/8
    x = np.log(np.float64([4.0, 8.0, 1.0, 2.0]))           # vocabulary order: 1/2, 1, 1/8, 1/4
    # top_k = 2 keeps tokens 1 and 0, masses 1 and 1/2: CDF in index order 1/3 | 1
    assert _one(oracle, x, 1.0, 1.0, 0.30, top_k=2) == (0, 2)
    assert _one(oracle, x, 1.0, 1.0, 0.34, top_k=2) == (1, 2)
    # min_p = 0.2 drops only the 1/8 token: masses (index order) 1/2, 1, -, 1/4 of 7/4
    assert _one(oracle, x, 1.0, 1.0, 0.28, min_p=0.2) == (0, 3)
    assert _one(oracle, x, 1.0, 1.0, 0.29, min_p=0.2) == (1, 3)
    assert _one(oracle, x, 1.0, 1.0, 0.86, min_p=0.2) == (3, 3)
    # either side of the 1/4 token
    assert _one(oracle, x, 1.0, 1.0, 0.99, min_p=0.24) == (3, 3)
    assert _one(oracle, x, 1.0, 1.0, 0.99, min_p=0.26) == (1, 2)
    # a probability exactly on the threshold stays (>=): the maximum itself at min_p = 1
    assert _one(oracle, x, 1.0, 1.0, 0.5, min_p=1.0) == (1, 1)
    # top_k = 3 then top_p = 0.6 over the survivors' mass 7/4: need 1.05 -> 1 + 1/2 reaches it: two kept
    assert _one(oracle, x, 1.0, 0.6, 0.99, top_k=3) == (1, 2)
    # without top_k the same top_p works on mass 15/8: need 1.125 -> still two kept
    assert _one(oracle, x, 1.0, 0.6, 0.99) == (1, 2)
    # top_p = 0.9: of 7/4 -> need 1.575 -> three kept; of 15/8 -> need 1.6875 -> three kept (1.75 >= 1.6875)
    assert _one(oracle, x, 1.0, 0.9, 0.999, top_k=3)[1] == 3
    assert _one(oracle, x, 1.0, 0.9, 0.999)[1] == 3
    # temperature acts before the filters: at T = 0.5 the probabilities are 1, 1/4, 1/16, 1/64
    assert _one(oracle, x, 0.5, 1.0, 0.5, min_p=0.2)[1] == 2


def test_ties_with_the_kth_are_kept(oracle):
    x = np.float32([1.0, 3.0, 1.0, 1.0, 0.0])
    assert _one(oracle, x, 1.0, 1.0, 0.999, top_k=2) == (3, 4)   # the three 1.0s tie for second place
    assert _one(oracle, x, 1.0, 1.0, 0.999, top_k=1) == (1, 1)


def test_kept_set_is_nested(oracle):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((1, 500)) * 3).astype(np.float32)
    prev = 0
    for k in (1, 2, 5, 17, 100, 499, 500, 900):
        kept = _one(oracle, x[0], 0.8, 1.0, 0.5, top_k=k)[1]
        assert prev <= kept <= min(k, 500) or kept >= k   # ties may exceed k, never shrink
        assert kept >= prev
        prev = kept
    prev = 500
    for mp in (1e-9, 1e-4, 1e-2, 0.1, 0.5, 1.0):
        kept = _one(oracle, x[0], 0.8, 1.0, 0.5, min_p=mp)[1]
        assert kept <= prev
        prev = kept


def _brute(x, T, top_p, u, top_k, min_p):
    x = np.asarray(x, dtype=np.float64)
    p = np.exp((x - x.max()) / T)
    alive = np.ones(len(x), bool)
    if min_p > 0:
        alive &= p >= min_p
    if top_k > 0 and alive.sum() > top_k:
        kth = np.sort(p[alive])[::-1][top_k - 1]
        alive &= p >= kth
    if top_p < 1:
        need = top_p * p[alive].sum()
        best = None
        for t in sorted(set(p[alive]), reverse=True):      # largest value whose upper set reaches need
            if p[alive & (p >= t)].sum() >= need:
                best = t
                break
        alive &= p >= best
    z = p[alive].sum()
    c = 0.0
    last = None
    for i in range(len(x)):
        if alive[i]:
            last = i
            c += p[i]
            if c > u * z:
                return i, int(alive.sum())
    return last, int(alive.sum())


def test_brute_force_on_tiny_vocabularies(oracle):
    rng = np.random.default_rng(4)
    for trial in range(300):
        v = int(rng.integers(1, 9))
        x = np.round(rng.standard_normal(v) * 2, 1).astype(np.float32)   # coarse values: ties happen
        T = float(rng.choice([0.5, 1.0, 2.0]))
        tp = float(rng.choice([0.3, 0.6, 0.9, 1.0]))
        k = int(rng.choice([0, 1, 2, 3, 8]))
        mp = float(rng.choice([0.0, 0.05, 0.3, 0.9]))
        u = float(rng.random())
        got = _one(oracle, x, T, tp, u, top_k=k, min_p=mp)
        want = _brute(x, T, tp, np.float32(u), k, np.float32(mp) if mp else 0.0)
        assert got == want, (trial, x, T, tp, k, mp, u, got, want)


def _full(oracle, x, T, top_p, u, top_k=0, min_p=0.0):
    x = np.asarray([x], dtype=np.float32)
    r = oracle.sample_tokens_filtered(x, np.float32([T]), np.float32([top_p]), np.float32([u]),
                                      np.int32([top_k]), np.float32([min_p]))
    return {k: v[0] for k, v in r.items()}


def f32(v):
    """The value the checker sees for a float32 parameter."""
    return float(np.float32(v))


def test_margins_closed_forms(oracle):
    """The margins decide which rows a GPU parity test may exempt, so they are pinned to closed
    forms on the four-token row p = 1/2, 1, 1/8, 1/4 (vocabulary order): a margin stuck at 0, at
    inf, or measured against the wrong neighbour fails here."""
    x = np.log(np.float64([4.0, 8.0, 1.0, 2.0]))
    # no filter acts: nothing to be near to
    r = _full(oracle, x, 1.0, 1.0, 0.5)
    assert np.isinf(r["filter_margin"]) and np.isinf(r["cut_margin"])
    # top_k >= the number of tokens removes nothing either
    assert np.isinf(_full(oracle, x, 1.0, 1.0, 0.5, top_k=4)["filter_margin"])
    # min_p = 0.24: the nearest probability is 1/4 -> |0.25 - 0.24| / 0.24
    r = _full(oracle, x, 1.0, 1.0, 0.5, min_p=0.24)
    assert abs(r["filter_margin"] - (0.25 - f32(0.24)) / f32(0.24)) < 1e-6
    # min_p = 0.26 is as near to 1/4 from the other side
    r = _full(oracle, x, 1.0, 1.0, 0.5, min_p=0.26)
    assert abs(r["filter_margin"] - (f32(0.26) - 0.25) / f32(0.26)) < 1e-6
    # min_p exactly on a probability (the maximum has p = 1 exactly): tokens on the threshold are not
    # counted (distance 0) and stay; the nearest other probability is 1/2 -> margin 1/2
    r = _full(oracle, np.float64([0.0, 0.0, np.log(0.5)]), 1.0, 1.0, 0.5, min_p=1.0)
    assert abs(r["filter_margin"] - 0.5) < 1e-6 and r["kept"] == 2
    # top_k = 2: tau_k = 1/2, the next smaller probability is 1/4 -> (1/2 - 1/4) / (1/2)
    r = _full(oracle, x, 1.0, 1.0, 0.5, top_k=2)
    assert abs(r["filter_margin"] - 0.5) < 1e-6
    # top_k = 3: tau_k = 1/4, next 1/8 -> 1/2 again; top_k = 1: tau_k = 1, next 1/2 -> 1/2
    assert abs(_full(oracle, x, 1.0, 1.0, 0.5, top_k=3)["filter_margin"] - 0.5) < 1e-6
    # both filters: the smaller of the two margins
    r = _full(oracle, x, 1.0, 1.0, 0.5, top_k=2, min_p=0.12)
    assert abs(r["filter_margin"] - (0.125 - f32(0.12)) / f32(0.12)) < 1e-6
    # unequal gaps tell the neighbours apart: p = 1, 0.9, 0.5 (index order 0.9, 1, 0.5), top_k = 2
    y = np.log(np.float64([0.9, 1.0, 0.5]))
    r = _full(oracle, y, 1.0, 1.0, 0.5, top_k=2)
    assert abs(r["filter_margin"] - (0.9 - 0.5) / 0.9) < 1e-6
    r = _full(oracle, y, 1.0, 1.0, 0.5, top_k=1)
    assert abs(r["filter_margin"] - 0.1) < 1e-6


def test_cut_margin_and_cdf_interval_of_the_filtered_rule(oracle):
    x = np.log(np.float64([4.0, 8.0, 1.0, 2.0]))
    # top_k = 3 leaves masses 1, 1/2, 1/4 (S2 = 7/4); top_p = 0.6 needs 1.05: running mass 1 then 3/2
    # -> margin = min(|1 - 1.05|, |1.5 - 1.05|) / 1.75
    r = _full(oracle, x, 1.0, 0.6, 0.99, top_k=3)
    assert abs(r["cut_margin"] - abs(1.0 - f32(0.6) * 1.75) / 1.75) < 1e-6
    # without top_k the same cut is measured against S = 15/8
    r = _full(oracle, x, 1.0, 0.6, 0.99)
    assert abs(r["cut_margin"] - abs(1.0 - f32(0.6) * 1.875) / 1.875) < 1e-6
    # top_k = 2: kept masses in index order 1/2, 1 of 3/2 -> token 0 owns [0, 1/3), token 1 [1/3, 1)
    r = _full(oracle, x, 1.0, 1.0, 0.30, top_k=2)
    assert r["token"] == 0 and r["cdf_lo"] == 0.0 and abs(r["cdf_hi"] - 1.0 / 3.0) < 1e-6
    r = _full(oracle, x, 1.0, 1.0, 0.34, top_k=2)
    assert r["token"] == 1 and abs(r["cdf_lo"] - 1.0 / 3.0) < 1e-6 and abs(r["cdf_hi"] - 1.0) < 1e-6
    # min_p = 0.2 drops the 1/8 token: intervals 2/7 | 6/7 | 1
    r = _full(oracle, x, 1.0, 1.0, 0.5, min_p=0.2)
    assert r["token"] == 1 and abs(r["cdf_lo"] - 2.0 / 7.0) < 1e-6 and abs(r["cdf_hi"] - 6.0 / 7.0) < 1e-6
