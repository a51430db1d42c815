"""Pins for the must-keep rules and the set part of the selection (Sec. 3.3; Alg. 1 step 5)."""
import os

import numpy as np

from paper_2605_23200_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example_must_keep.txt")


def _read(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = np.array([float(x) for x in v])
    return out


def _topk_lower_index_first(g, cand, k):
    """The k candidates with the largest g, equal scores by lower index (plain numpy)."""
    cand = np.asarray(sorted(cand), dtype=np.int64)
    order = np.argsort(-g[cand].astype(np.float64), kind="stable")
    return set(cand[order[:k]].tolist())


def test_worked_example(oracle):
    w = _read(GOLD)
    g = w["g"].astype(np.float32)
    T = len(g)
    se, le, sb = oracle.must_keep(T, int(w["budget"][0]), int(w["n_sink"][0]), int(w["n_last"][0]))
    assert (se, le, sb) == (int(w["sink_eff"][0]), int(w["last_eff"][0]), int(w["seg_budget"][0]))
    q = oracle.quota(w["bounds"].astype(np.int32), w["seg_mass"].astype(np.float32), sb, int(w["q_min"][0]))
    np.testing.assert_array_equal(q, w["quota"].astype(np.int32))
    seg = oracle.select(g, w["bounds"].astype(np.int32), q)
    np.testing.assert_array_equal(seg, w["seg_idx"].astype(np.int32))
    idx = oracle.finalize(g, seg, se, le, min(int(w["budget"][0]), T))
    np.testing.assert_array_equal(idx, w["idx"].astype(np.int32))


def test_must_keep_sizes(oracle):
    assert oracle.must_keep(100, 20, 4, 8) == (4, 8, 8)
    assert oracle.must_keep(100, 20, 0, 0) == (0, 0, 20)
    assert oracle.must_keep(100, 10, 4, 8) == (4, 6, 0)        # the recent suffix gives way
    assert oracle.must_keep(100, 3, 4, 8) == (3, 0, 0)         # sinks alone already fill the budget
    assert oracle.must_keep(6, 20, 4, 8) == (4, 2, 0)          # short cache: everything is kept anyway
    assert oracle.must_keep(5, 4, 2, 1) == (2, 1, 1)


def test_finalize_without_must_keep_is_the_identity(oracle):
    rng = np.random.default_rng(3)
    for _ in range(50):
        T = int(rng.integers(4, 80))
        g = rng.standard_normal(T).astype(np.float32)
        n = int(rng.integers(1, T + 1))
        seg = np.sort(rng.choice(T, n, replace=False)).astype(np.int32)
        np.testing.assert_array_equal(oracle.finalize(g, seg, 0, 0, n), seg)


def test_quota_of_zero_budget(oracle):
    q = oracle.quota(np.array([0, 5, 9], np.int32), np.array([0.5, 0.5], np.float32), 0, 1)
    np.testing.assert_array_equal(q, [0, 0])


def test_one_segment_is_must_keep_plus_global_topk_of_the_rest(oracle):
    # with a single segment the in-segment pick is a global top-k; what it spends on must-keep
    # positions comes back through the backfill, so the result is must + best of the others
    rng = np.random.default_rng(5)
    for trial in range(60):
        T = int(rng.integers(8, 200))
        g = rng.standard_normal(T).astype(np.float32)
        if trial % 3 == 0:
            g = np.round(g * 2) / 2                              # many equal scores
        budget = int(rng.integers(1, T + 10))
        n_sink, n_last = int(rng.integers(0, 6)), int(rng.integers(0, 12))
        se, le, sb = oracle.must_keep(T, budget, n_sink, n_last)
        bounds = np.array([0, T], np.int32)
        q = oracle.quota(bounds, np.array([1.0], np.float32), sb, 1)
        seg = oracle.select(g, bounds, q)
        idx = oracle.finalize(g, seg, se, le, min(budget, T))
        must = set(range(se)) | set(range(T - le, T))
        want = must | _topk_lower_index_first(g, set(range(T)) - must, min(budget, T) - len(must))
        assert idx.tolist() == sorted(want)


def test_set_invariants_with_segments(oracle):
    rng = np.random.default_rng(7)
    for _ in range(60):
        T = int(rng.integers(20, 400))
        S = int(rng.integers(1, 9))
        g = rng.random(T).astype(np.float32)
        m = rng.random(T).astype(np.float32) ** 4 + 1e-6
        m = (m / m.sum()).astype(np.float32)
        bounds, seg_mass = oracle.segment(m, S)
        budget = int(rng.integers(1, T))
        n_sink, n_last = int(rng.integers(0, 6)), int(rng.integers(0, 40))
        se, le, sb = oracle.must_keep(T, budget, n_sink, n_last)
        q = oracle.quota(bounds, seg_mass, sb, 1)
        assert q.sum() == sb
        seg = oracle.select(g, bounds, q)
        idx = oracle.finalize(g, seg, se, le, budget)
        assert len(idx) == budget and np.all(np.diff(idx) > 0)
        kept = set(idx.tolist())
        must = set(range(se)) | set(range(T - le, T))
        assert must <= kept and set(seg.tolist()) <= kept
        filled = kept - must - set(seg.tolist())
        assert len(filled) == budget - len(must | set(seg.tolist()))
        rest = np.array(sorted(set(range(T)) - kept), dtype=np.int64)
        if filled and len(rest):
            assert min(g[t] for t in filled) >= g[rest].max()     # backfill took the best of what was left


def test_trim_drops_lowest_scores_outside_the_must_keep_set(oracle):
    rng = np.random.default_rng(9)
    for trial in range(40):
        T = int(rng.integers(10, 120))
        g = rng.standard_normal(T).astype(np.float32)
        if trial % 2:
            g = np.round(g)
        se, le = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        n = int(rng.integers(1, T + 1))
        seg = rng.choice(T, n, replace=False).astype(np.int32)
        must = set(range(se)) | set(range(T - le, T))
        union = must | set(seg.tolist())
        target = int(rng.integers(len(must), len(union) + 1))
        if target < 1:
            continue
        idx = oracle.finalize(g, seg, se, le, target)
        want = must | _topk_lower_index_first(g, union - must, target - len(must))
        assert idx.tolist() == sorted(want)


def test_whole_event_with_must_keep(oracle):
    w = inputs.CONFIGS[0].scaled(T=600, budget=96, S=8, n_spans=3, span_len=(16, 48), H=1)
    q = inputs.unit_q(w, 0, 0, 0)
    k, v = inputs.unit_kv(w, 0, 0, 0, w.T, q)
    kw = dict(G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam)
    plain = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), **kw)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), n_sink=4, n_last=16, **kw)
    # scores, mass and segments do not depend on the must-keep set
    for key in ("u", "g", "m_used", "bounds", "seg_mass"):
        np.testing.assert_array_equal(r[key], plain[key])
    assert r["quota"].sum() == w.budget - 20
    seg = oracle.select(r["g"], r["bounds"], r["quota"])
    np.testing.assert_array_equal(r["idx"], oracle.finalize(r["g"], seg, 4, 16, w.budget))
    assert r["n_kept"] == w.budget
    assert set(range(4)) <= set(r["idx"].tolist()) and set(range(w.T - 16, w.T)) <= set(r["idx"].tolist())
    np.testing.assert_array_equal(r["K_out"], k[r["idx"]])
    np.testing.assert_array_equal(r["credit_out"], r["credit"][r["idx"]])
    # a must-keep set larger than the budget: sinks and as much of the suffix as fits, nothing else
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), n_sink=4, n_last=200, **kw)
    assert r["idx"].tolist() == list(range(4)) + list(range(w.T - 92, w.T))
