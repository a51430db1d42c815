"""Pins for quota allocation and in-segment top-k of the oracle (Sec. 3.3; Alg. 1 steps 4-5)."""
import itertools

import numpy as np
import pytest


def _bounds(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def test_quota_sums_to_budget_and_respects_lengths(oracle):
    rng = np.random.default_rng(0)
    for _ in range(300):
        S = int(rng.integers(1, 12))
        lengths = rng.integers(0, 40, size=S)
        if lengths.sum() == 0:
            lengths[0] = 3
        mass = rng.random(S).astype(np.float32) ** 3
        mass[lengths == 0] = 0
        budget = int(rng.integers(1, 2 * lengths.sum() + 1))
        qmin = int(rng.integers(0, 4))
        q = oracle.quota(_bounds(lengths), mass, budget, qmin)
        assert q.sum() == min(budget, lengths.sum())
        assert np.all(q >= 0) and np.all(q <= lengths)
        need = np.minimum(qmin, lengths).sum()
        if need <= budget:
            assert np.all(q >= np.minimum(qmin, lengths))        # no region wiped out


def test_quota_equal_segments_get_equal_shares(oracle):
    q = oracle.quota(_bounds([512] * 8), np.full(8, 0.125, np.float32), 1024, 1)
    np.testing.assert_array_equal(q, [128] * 8)


def test_quota_is_largest_remainder_when_no_cap_binds(oracle):
    # Hamilton apportionment of 10 seats to shares .43 .33 .24 (q_min = 0): quotas 4.3 3.3 2.4 ->
    # integer parts 4 3 2, the one left over goes to the largest remainder (.4) -> 4 3 3
    q = oracle.quota(_bounds([100, 100, 100]), np.array([0.43, 0.33, 0.24], np.float32), 10, 0)
    np.testing.assert_array_equal(q, [4, 3, 3])
    # with q_min = 1 the remainder 7 is shared: 3.01 2.31 1.68 -> 3 2 1 + leftover to .68 -> 4 3 3
    q = oracle.quota(_bounds([100, 100, 100]), np.array([0.43, 0.33, 0.24], np.float32), 10, 1)
    np.testing.assert_array_equal(q, [4, 3, 3])


def test_quota_caps_and_redistributes(oracle):
    # segment 0 holds 90% of the mass but only 4 tokens: it is filled, the rest is re-shared 1:1
    q = oracle.quota(_bounds([4, 50, 50]), np.array([0.9, 0.05, 0.05], np.float32), 24, 1)
    np.testing.assert_array_equal(q, [4, 10, 10])


def test_quota_budget_below_minimum(oracle):
    # 5 non-empty segments, budget 3 < 5 * q_min: the floor drops to 0 and mass decides
    q = oracle.quota(_bounds([10] * 5), np.array([0.4, 0.3, 0.2, 0.06, 0.04], np.float32), 3, 1)
    assert q.sum() == 3
    np.testing.assert_array_equal(q, [1, 1, 1, 0, 0])


def test_quota_budget_at_least_length_keeps_everything(oracle):
    lengths = [3, 0, 7, 1]
    q = oracle.quota(_bounds(lengths), np.array([0.1, 0, 0.8, 0.1], np.float32), 50, 1)
    np.testing.assert_array_equal(q, lengths)


def test_quota_brute_force_closest_to_proportional(oracle):
    # among all integer vectors x with sum x = R, 0 <= x_i <= room_i the oracle's allocation above the
    # floor is closest to the proportional shares of the final round (max and total deviation).
    rng = np.random.default_rng(1)
    for _ in range(120):
        S = int(rng.integers(2, 5))
        lengths = rng.integers(1, 8, size=S)
        mass = (rng.integers(1, 9, size=S) / 16).astype(np.float32)
        budget = int(rng.integers(S, min(12, lengths.sum()) + 1))
        q = oracle.quota(_bounds(lengths), mass, budget, 1)
        # replay the saturation rounds to know which segments were still sharing at the end
        room = lengths - 1
        active = room > 0
        rem = budget - S
        while True:
            if not active.any() or rem <= 0:
                break
            raw = rem * mass.astype(np.float64) / mass[active].astype(np.float64).sum()
            sat = active & (raw >= room)
            if not sat.any():
                break
            rem -= room[sat].sum()
            active &= ~sat
        for i in range(S):
            if not active[i]:
                assert q[i] == (lengths[i] if room[i] > 0 else 1) or rem <= 0
        if rem <= 0 or not active.any():
            continue
        ids = np.flatnonzero(active)
        x = (q - 1)[ids]
        assert x.sum() == rem
        best_max, best_sum = None, None
        for cand in itertools.product(*[range(room[i] + 1) for i in ids]):
            if sum(cand) != rem:
                continue
            dev = np.abs(np.array(cand) - raw[ids])
            if best_max is None or dev.max() < best_max - 1e-12:
                best_max = dev.max()
            if best_sum is None or dev.sum() < best_sum - 1e-12:
                best_sum = dev.sum()
        dev = np.abs(x - raw[ids])
        assert dev.max() <= best_max + 1e-9
        assert dev.sum() <= best_sum + 1e-9


def test_select_takes_exactly_the_quota_per_segment(oracle):
    rng = np.random.default_rng(2)
    g = rng.standard_normal(200).astype(np.float32)
    bounds = np.array([0, 10, 10, 75, 199, 200], np.int32)
    quota = np.array([3, 0, 20, 5, 1], np.int32)
    idx = oracle.select(g, bounds, quota)
    assert len(idx) == quota.sum() and np.all(np.diff(idx) > 0)
    for i in range(5):
        inside = idx[(idx >= bounds[i]) & (idx < bounds[i + 1])]
        assert len(inside) == quota[i]
        seg = g[bounds[i]:bounds[i + 1]]
        if quota[i]:
            assert g[inside].min() >= np.sort(seg)[::-1][quota[i] - 1]


def test_single_segment_is_global_topk(oracle):
    g = np.random.default_rng(3).standard_normal(500).astype(np.float32)
    g[100:140] = g[7]                     # plenty of ties
    k = 60
    idx = oracle.select(g, np.array([0, 500], np.int32), np.array([k], np.int32))
    order = np.argsort(-g.astype(np.float64), kind="stable")      # ties keep the lower index first
    np.testing.assert_array_equal(idx, np.sort(order[:k]))


def test_all_equal_scores_keep_first_positions(oracle):
    idx = oracle.select(np.zeros(30, np.float32), np.array([0, 10, 30], np.int32), np.array([4, 3], np.int32))
    np.testing.assert_array_equal(idx, [0, 1, 2, 3, 10, 11, 12])


def test_signed_zero_ties_and_nan_is_lowest(oracle):
    g = np.array([-0.0, 0.0, -0.0, 1.0], np.float32)
    np.testing.assert_array_equal(oracle.select(g, np.array([0, 4], np.int32), np.array([2], np.int32)), [0, 3])
    g = np.array([np.nan, -np.inf, -5.0, np.nan], np.float32)
    np.testing.assert_array_equal(oracle.select(g, np.array([0, 4], np.int32), np.array([2], np.int32)), [0, 2])
    np.testing.assert_array_equal(oracle.select(g, np.array([0, 4], np.int32), np.array([3], np.int32)), [0, 1, 2])


def test_select_brute_force_best_sum_and_lexicographically_first(oracle):
    rng = np.random.default_rng(4)
    for _ in range(60):
        T = int(rng.integers(4, 12))
        g = rng.integers(-2, 3, size=T).astype(np.float32)          # few distinct values -> many ties
        cut = int(rng.integers(1, T))
        bounds = np.array([0, cut, T], np.int32)
        quota = np.array([rng.integers(0, cut + 1), rng.integers(0, T - cut + 1)], np.int32)
        idx = oracle.select(g, bounds, quota)
        best = None
        for a in itertools.combinations(range(0, cut), int(quota[0])):
            for b in itertools.combinations(range(cut, T), int(quota[1])):
                cand = a + b
                key = (-float(g[list(cand)].sum()) if cand else 0.0, cand)
                if best is None or key < best:
                    best = key
        assert tuple(idx) == best[1]
