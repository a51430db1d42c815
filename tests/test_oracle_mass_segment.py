"""Pins for Eq. (1), the EMA credit and the prefix-sum segmentation of the oracle (Sec. 3.2, 3.3)."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = [float(x) for x in v]
    return out


def test_worked_example_mass_bounds_quota_select(oracle):
    gold = _load("worked_example_T8.txt")
    u = np.array(gold["u"], np.float32)
    S, bud, qmin = int(gold["S"][0]), int(gold["budget"][0]), int(gold["q_min"][0])
    m = oracle.mass(u, gold["eps"][0])
    np.testing.assert_array_equal(m, np.array(gold["m"], np.float32))
    bounds, seg_mass = oracle.segment(m, S)
    np.testing.assert_array_equal(bounds, np.array(gold["bounds"], np.int32))
    np.testing.assert_array_equal(seg_mass, np.array(gold["seg_mass"], np.float32))
    q = oracle.quota(bounds, seg_mass, bud, qmin)
    np.testing.assert_array_equal(q, np.array(gold["quota"], np.int32))
    idx = oracle.select(u, bounds, q)
    np.testing.assert_array_equal(idx, np.array(gold["idx"], np.int32))


def test_worked_example_ema(oracle):
    gold = _load("worked_example_ema.txt")
    m = np.array(gold["m_cur"], np.float32)
    m_used, c = oracle.ema(m, np.array(gold["credit"], np.float32), gold["lambda"][0], gold["beta"][0])
    np.testing.assert_array_equal(c, np.array(gold["credit_new"], np.float32))
    np.testing.assert_array_equal(m_used, np.array(gold["m_used"], np.float32))
    m_used, c = oracle.ema(m, np.array(gold["credit2"], np.float32), 0.5, 0.5)
    np.testing.assert_array_equal(c, np.array(gold["credit2_new"], np.float32))
    want = np.array([float(Fraction(int(n), int(gold["m_used2_den"][0]))) for n in gold["m_used2_num"]])
    np.testing.assert_allclose(m_used, want, rtol=1.2e-7)


def test_mass_sums_to_one_and_is_positive(oracle):
    u = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    m = oracle.mass(u, 1e-6)
    assert abs(m.astype(np.float64).sum() - 1) < 1e-6
    assert (m > 0).all()
    # negative usage contributes only eps
    assert np.all(m[u <= 0] == m[u <= 0][0])


def test_mass_uniform_when_usage_nonpositive(oracle):
    m = oracle.mass(-np.abs(np.random.default_rng(1).standard_normal(64)).astype(np.float32), 1e-3)
    np.testing.assert_array_equal(m, np.full(64, 1 / 64, np.float32))


def test_ema_lambda_zero_is_identity(oracle):
    m = oracle.mass(np.random.default_rng(2).random(257).astype(np.float32))
    m_used, c = oracle.ema(m, np.random.default_rng(3).random(257).astype(np.float32), 0.0, 0.3)
    np.testing.assert_array_equal(m_used, m)
    np.testing.assert_array_equal(c, m)


def test_ema_beta_one_ignores_credit(oracle):
    m = oracle.mass(np.random.default_rng(4).random(300).astype(np.float32))
    m_used, _ = oracle.ema(m, np.random.default_rng(5).random(300).astype(np.float32), 0.9, 1.0)
    np.testing.assert_allclose(m_used, m, rtol=3e-7)


def test_ema_constant_mass_follows_geometric_series(oracle):
    # c_e = (1 - lambda^e) m from zero credit, so normalize(c) = m and m_used = m at every event
    m = oracle.mass(np.random.default_rng(6).random(128).astype(np.float32))
    c = np.zeros(128, np.float32)
    lam = 0.75
    for e in range(1, 6):
        m_used, c = oracle.ema(m, c, lam, 0.4)
        np.testing.assert_allclose(c, (1 - lam ** e) * m.astype(np.float64), rtol=1e-6)
        np.testing.assert_allclose(m_used, m, rtol=1e-6)


def test_ema_history_pulls_mass_towards_credit(oracle):
    m = np.array([0.25, 0.25, 0.25, 0.25], np.float32)
    m_used, _ = oracle.ema(m, np.array([1, 0, 0, 0], np.float32), 0.5, 0.5)
    assert m_used[0] > m_used[1] == m_used[2] == m_used[3]
    assert abs(float(m_used.sum()) - 1) < 1e-6


def test_uniform_mass_gives_equal_segments(oracle):
    T, S = 4096, 8
    bounds, seg_mass = oracle.segment(np.full(T, 1 / T, np.float32), S)
    np.testing.assert_array_equal(bounds, np.arange(S + 1) * (T // S))
    np.testing.assert_array_equal(seg_mass, np.full(S, 1 / S, np.float32))


def test_spike_collapses_boundaries(oracle):
    T, S = 100, 5
    m = np.full(T, 1e-9, np.float32)
    m[40] = 1.0
    bounds, seg_mass = oracle.segment(m, S)
    np.testing.assert_array_equal(bounds, [0, 41, 41, 41, 41, 100])
    assert seg_mass[1] == seg_mass[2] == seg_mass[3] == 0


def test_bracket_invariant_on_random_mass(oracle):
    rng = np.random.default_rng(7)
    for T, S in ((1000, 16), (333, 7), (50, 64), (5, 3), (1, 4)):
        m = oracle.mass(rng.random(T).astype(np.float32) ** 4)
        bounds, seg_mass = oracle.segment(m, S)
        assert bounds[0] == 0 and bounds[S] == T and np.all(np.diff(bounds) >= 0)
        c = np.cumsum(m.astype(np.float64))
        for k in range(1, S):
            e = bounds[k]
            if e == T and c[T - 1] < k / S:
                continue
            assert c[e - 1] >= k / S
            assert e < 2 or c[e - 2] < k / S or bounds[k - 1] == e
        for i in range(S):
            np.testing.assert_allclose(seg_mass[i], m[bounds[i]:bounds[i + 1]].astype(np.float64).sum(),
                                       rtol=1e-6, atol=1e-12)


def test_threshold_never_reached_gives_T(oracle):
    # total mass below 1: upper thresholds are never crossed
    bounds, _ = oracle.segment(np.full(10, 0.05, np.float32), 4)
    np.testing.assert_array_equal(bounds, [0, 5, 10, 10, 10])
