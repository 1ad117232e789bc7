"""Pins for the fp64 sampling checker: hand-worked closed forms (tests/golden),
limits, monotonicity, frequency counts and a second, sort-free formulation.
The paper fixes only the temperature (App. "Experiment settings"); the nucleus
and inverse-CDF rule are stated in the checker's header."""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sampler_closed_forms.txt")


def _one(oracle, logits, T, top_p, u):
    r = oracle.sample_tokens(np.asarray([logits], np.float32), [T], [top_p], [u])
    return {k: v[0] for k, v in r.items()}


def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        probs, T, top_p, u, tok = [c.strip() for c in line.split("|")]
        cases.append(([float(x) for x in probs.split(",")], float(T), float(top_p), float(u), int(tok)))
    return cases


@pytest.mark.parametrize("probs,T,top_p,u,tok", _golden_cases())
def test_hand_worked_cases(oracle, probs, T, top_p, u, tok):
    logits = [math.log(p) for p in probs]
    assert _one(oracle, logits, T, top_p, u)["token"] == tok


def test_two_token_boundary_values(oracle):
    r = _one(oracle, [math.log(3.0), 0.0], 1.0, 1.0, 0.9)
    assert r["token"] == 1 and abs(r["cdf_lo"] - 0.75) < 1e-7 and abs(r["cdf_hi"] - 1.0) < 1e-12
    r = _one(oracle, [math.log(0.5), math.log(0.3), math.log(0.2)], 1.0, 0.7, 0.7)
    assert r["token"] == 1 and abs(r["cdf_lo"] - 0.625) < 1e-7 and r["kept"] == 2
    assert abs(r["cut_margin"] - 0.1) < 1e-6       # |0.8 - 0.7| and |0.5 - 0.7| -> 0.1


def test_equal_logits_give_floor_uV(oracle):
    V = 1000
    for top_p in (1.0, 0.3):                       # ties with the threshold are all kept
        for u in (0.0, 0.0005, 0.1234, 0.5, 0.99951):
            tok = _one(oracle, np.full(V, 1.7), 0.9, top_p, u)["token"]
            assert tok == int(math.floor(np.float32(u).astype(np.float64) * V))


def test_limits_give_argmax(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal(500).astype(np.float32) * 3
    am = int(np.argmax(x))
    assert _one(oracle, x, 1e-4, 1.0, 0.73)["token"] == am        # T -> 0+
    assert _one(oracle, x, 1.0, 1e-9, 0.73)["token"] == am        # top_p -> 0+
    x[[100, 40, 300]] = x.max() + 1
    assert _one(oracle, x, 0.0, 0.5, 0.99)["token"] == 40         # T == 0: lowest index of the maximum


def test_token_is_monotone_in_u(oracle):
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(300) * 3).astype(np.float32)
    us = np.sort(rng.random(400).astype(np.float32))
    r = oracle.sample_tokens(np.tile(x, (400, 1)), np.full(400, 0.7), np.full(400, 0.9), us)
    assert np.all(np.diff(r["token"]) >= 0)
    assert np.all(r["cdf_lo"] <= us + 1e-12) and np.all(us < r["cdf_hi"] + 1e-12)


def test_stratified_uniforms_reproduce_the_distribution(oracle):
    x = np.array([0.3, -1.0, 2.0, 0.0, 1.1, -0.4, 0.9, -2.5], np.float32)
    T, top_p, M = 0.8, 0.9, 200000
    us = ((np.arange(M) + 0.5) / M).astype(np.float32)
    r = oracle.sample_tokens(np.tile(x, (M, 1)), np.full(M, T), np.full(M, top_p), us)
    p = np.exp((x.astype(np.float64) - x.max()) / np.float32(T).astype(np.float64))
    order = np.argsort(-p)
    c = np.cumsum(p[order])
    k = np.searchsorted(c, np.float32(top_p).astype(np.float64) * p.sum())
    kept = np.zeros(8, bool)
    kept[order[: k + 1]] = True
    expect = np.where(kept, p, 0) / p[kept].sum() * M
    counts = np.bincount(r["token"], minlength=8)
    assert np.all(counts[~kept] == 0)
    assert np.all(np.abs(counts - expect) <= 2.0)


def _threshold_formulation(x, T, top_p, u):
    """The rule written without ordering the row: tau is the largest value t among the p_i whose
    upper set {p_i >= t} has mass >= top_p * S (each upper-set mass is a masked sum over the
    vocabulary, distinct values visited in no particular order); then the index-order walk."""
    x = np.asarray(x, np.float32).astype(np.float64)
    T, top_p, u = (float(np.float32(v)) for v in (T, top_p, u))
    p = np.exp((x - x.max()) / T)
    S = float(p.sum())
    tau = 0.0
    if top_p < 1.0:
        reaching = [t for t in set(p.tolist()) if float(np.where(p >= t, p, 0.0).sum()) >= top_p * S]
        tau = max(reaching) if reaching else float(p.min())
    kept = p >= tau
    Z = float(np.where(kept, p, 0.0).sum())
    running = np.cumsum(np.where(kept, p, 0.0))
    hit = np.nonzero(kept & (running > u * Z))[0]
    return int(hit[0]) if len(hit) else int(np.nonzero(kept)[0][-1])


def test_second_formulation_agrees_on_random_tiny_rows(oracle):
    rng = np.random.default_rng(7)
    for trial in range(200):
        V = int(rng.integers(2, 40))
        x = np.round(rng.standard_normal(V) * 3, 1).astype(np.float32)        # rounding makes ties common
        T = float(rng.choice([0.2, 0.4, 0.7, 1.0, 1.2]))
        top_p = float(rng.choice([0.1, 0.5, 0.9, 0.95, 1.0]))
        u = float(rng.random())
        assert _one(oracle, x, T, top_p, u)["token"] == _threshold_formulation(x, T, top_p, u), (trial, x, T, top_p, u)


def test_shift_and_joint_scaling_invariance(oracle):
    rng = np.random.default_rng(9)
    x = np.round(rng.standard_normal((64, 200)) * 3 * 8) / 8        # multiples of 1/8: shifts and halving are exact
    us = rng.random(64).astype(np.float32)
    a = oracle.sample_tokens(x, np.full(64, 0.5), np.full(64, 0.9), us)
    b = oracle.sample_tokens(x + 4.0, np.full(64, 0.5), np.full(64, 0.9), us)
    c = oracle.sample_tokens(x * 0.5, np.full(64, 0.25), np.full(64, 0.9), us)
    np.testing.assert_array_equal(a["token"], b["token"])
    np.testing.assert_array_equal(a["token"], c["token"])
    np.testing.assert_allclose(a["cdf_lo"], c["cdf_lo"], atol=1e-14)


def test_u_zero_returns_first_kept_token_with_mass(oracle):
    x = np.array([-1000.0, -3.0, 2.0, 1.0], np.float32)          # p[0] underflows to exactly 0 at T = 1
    assert _one(oracle, x, 1.0, 1.0, 0.0)["token"] == 1
    assert _one(oracle, x, 1.0, 0.9, 0.0)["token"] == 2


def test_rows_are_independent_and_stride_respected(oracle):
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((5, 64)) * 3).astype(np.float32)
    t = np.array([0.4, 0.7, 1.0, 0.0, 1.2], np.float32)
    tp = np.array([0.9, 1.0, 0.5, 0.9, 0.95], np.float32)
    u = rng.random(5).astype(np.float32)
    full = oracle.sample_tokens(x, t, tp, u)["token"]
    for r in range(5):
        assert _one(oracle, x[r], t[r], tp[r], u[r])["token"] == full[r]
