"""Pins for the segmentation as printed (thresholds k*delta, split / merge) and the usage pooling
(Sec. 3.3 "Mass-based adaptive segmentation"; Alg. 1 steps 1 and 3; App. A)."""
import os

import numpy as np
import pytest

from paper_2605_23200_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example_adaptive_segments.txt")
GOLD2 = os.path.join(os.path.dirname(__file__), "golden", "worked_example_adaptive_segments_2.txt")


def _read(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = np.array([float(x) for x in v])
    return out


@pytest.mark.parametrize("gold", [GOLD, GOLD2], ids=["split_and_merge", "empty_run_of_short_and_overlong"])
def test_worked_example(oracle, gold):
    w = _read(gold)
    m = (w["m64"] / 64).astype(np.float32)
    cap = 12
    bounds, seg_mass, n = oracle.segment_adaptive(m, float(w["delta"][0]), int(w["l_min"][0]), int(w["l_max"][0]), cap)
    want = w["bounds"].astype(np.int32)
    assert n == len(want) - 1
    np.testing.assert_array_equal(bounds[: n + 1], want)
    assert (bounds[n + 1:] == len(m)).all() and (seg_mass[n:] == 0).all()
    np.testing.assert_array_equal(seg_mass[:n], (w["seg_mass64"] / 64).astype(np.float32))


@pytest.mark.parametrize("S", [1, 2, 4, 8, 16, 64])
def test_without_length_rules_equals_fixed_count_segmentation(oracle, S):
    # delta = 1/S exactly representable, no split / merge: the same cuts as the S-segment rule, minus empty segments
    rng = np.random.default_rng(S)
    for _ in range(20):
        T = int(rng.integers(S, 3000))
        m = oracle.mass((rng.random(T) ** 6).astype(np.float32))
        b_fixed, sm_fixed = oracle.segment(m, S)
        b, sm, n = oracle.segment_adaptive(m, 1.0 / S, 0, 0, S)
        keep = np.flatnonzero(np.diff(b_fixed) > 0)
        assert n == len(keep)
        np.testing.assert_array_equal(b[1: n + 1], b_fixed[keep + 1])
        np.testing.assert_array_equal(sm[:n], sm_fixed[keep])


def test_uniform_mass_closed_forms(oracle):
    T = 1024                                                               # 1/1024 is exact in binary
    m = np.full(T, 1.0 / T, np.float32)
    b, sm, n = oracle.segment_adaptive(m, 0.125, 0, 0, 16)                # 8 segments of 128
    assert n == 8
    np.testing.assert_array_equal(b[:9], np.arange(9) * 128)
    b, sm, n = oracle.segment_adaptive(m, 0.125, 0, 50, 64)               # each split into ceil(128/50) = 3: 43 43 42
    assert n == 24
    np.testing.assert_array_equal(np.diff(b[:25]), [43, 43, 42] * 8)
    np.testing.assert_allclose(sm[:24], np.array([43, 43, 42] * 8) / 1024, rtol=1e-6)
    # every initial segment (128) is shorter than L_min = 200: the first joins the second, each later one joins
    # the segment to its left, so one segment remains
    b, sm, n = oracle.segment_adaptive(m, 0.125, 200, 0, 16)
    assert n == 1 and b[1] == T and sm[0] == 1.0
    # L_min = 100 < 128: nothing to merge
    b, sm, n = oracle.segment_adaptive(m, 0.125, 100, 0, 16)
    assert n == 8
    # delta that does not divide 1: thresholds .3 .6 .9 -> cuts after 308, 615, 922 tokens (ceil(k*.3*1024)), 4 segments
    b, sm, n = oracle.segment_adaptive(m, 0.3, 0, 0, 8)
    assert n == 4
    np.testing.assert_array_equal(b[:5], [0, 308, 615, 922, 1024])


def test_invariants_on_random_masses(oracle):
    rng = np.random.default_rng(11)
    for _ in range(200):
        T = int(rng.integers(1, 2500))
        m = oracle.mass((rng.random(T) ** int(rng.integers(1, 12))).astype(np.float32))
        delta = float(rng.choice([0.5, 0.1, 0.05, 0.02, 0.3]))
        l_max = int(rng.choice([0, 16, 64, 256]))
        l_min = int(rng.choice([0, 4, 16])) if l_max != 16 else int(rng.choice([0, 4, 16]))
        cap = int(np.ceil(1 / delta)) + 1 + (T // l_max if l_max else 0)
        b, sm, n = oracle.segment_adaptive(m, delta, l_min, l_max, cap)
        assert 1 <= n <= cap
        assert b[0] == 0 and b[n] == T and np.all(np.diff(b[: n + 1]) > 0)      # a partition into non-empty segments
        np.testing.assert_allclose(sm[:n].sum(), 1.0, rtol=1e-5)
        for i in range(n):
            np.testing.assert_allclose(sm[i], m[b[i]:b[i + 1]].astype(np.float64).sum(), rtol=1e-6)
        lens = np.diff(b[: n + 1])
        if l_min == 0 and l_max > 0:
            assert lens.max() <= l_max                                           # only merging can exceed L_max
        if l_min > 0 and l_max == 0 and n > 1:
            assert lens.min() >= min(l_min, T)                                   # only ... nothing re-creates short ones
        # without the length rules every segment but the last holds at least delta minus one token's mass
        if l_min == 0 and l_max == 0:
            csum = np.cumsum(m.astype(np.float64))
            for i in range(n - 1):
                lo = csum[b[i] - 1] if b[i] > 0 else 0.0
                assert csum[b[i + 1] - 1] - lo > 0


def test_capacity_too_small_is_an_error(oracle):
    m = np.full(1024, 1.0 / 1024, np.float32)
    with pytest.raises(RuntimeError):
        oracle.segment_adaptive(m, 0.125, 0, 50, 8)


def test_pool_closed_forms(oracle):
    u = np.arange(10, dtype=np.float32)
    np.testing.assert_array_equal(oracle.pool(u, 1), u)
    # a linear ramp is its own centred mean in the interior; at the ends the window is cut
    p = oracle.pool(u, 3)
    np.testing.assert_allclose(p[1:-1], u[1:-1])
    np.testing.assert_allclose([p[0], p[-1]], [0.5, 8.5])
    p = oracle.pool(u, 5)
    np.testing.assert_allclose(p, [1.0, 1.5, 2, 3, 4, 5, 6, 7, 7.5, 8.0])
    # against numpy's convolution with the count of positions inside the sequence
    rng = np.random.default_rng(0)
    u = rng.random(200).astype(np.float32)
    for k in (3, 5, 7, 9):
        num = np.convolve(u.astype(np.float64), np.ones(k), mode="same")
        den = np.convolve(np.ones(200), np.ones(k), mode="same")
        np.testing.assert_allclose(oracle.pool(u, k), num / den, rtol=1e-6)
    # a spike is spread over k positions and the total is preserved away from the ends
    u = np.zeros(50, np.float32)
    u[20] = 1.0
    np.testing.assert_allclose(oracle.pool(u, 5)[18:23], 0.2)
    assert oracle.pool(u, 5).sum() == pytest.approx(1.0)


def test_whole_event_with_adaptive_segments_and_pooling(oracle):
    w = inputs.CONFIGS[0].scaled(T=900, budget=128, S=64, n_spans=3, span_len=(16, 48), H=1)
    q = inputs.unit_q(w, 0, 0, 0)
    k, v = inputs.unit_kv(w, 0, 0, 0, w.T, q)
    kw = dict(G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), delta=0.1, l_min=16, l_max=64, pool_kernel=5, **kw)
    u, g = oracle.score(q, k, w.G, w.W)
    np.testing.assert_array_equal(r["u"], u)                                   # the base score keeps the raw usage
    m_used, _ = oracle.ema(oracle.mass(oracle.pool(u, 5), w.eps), np.zeros(w.T, np.float32), w.lam, 0.9)
    np.testing.assert_array_equal(r["m_used"], m_used)
    b, sm, n = oracle.segment_adaptive(m_used, 0.1, 16, 64, w.S)
    np.testing.assert_array_equal(r["bounds"], b)
    np.testing.assert_array_equal(r["quota"], oracle.quota(b, sm, w.budget, 1))
    assert r["n_kept"] == w.budget and (r["quota"][:n] >= 1).all() and (r["quota"][n:] == 0).all()
