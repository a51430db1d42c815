"""Metric functions of the retention diagnostics (plain index-set arithmetic) and, on a GPU, a short
synthetic trajectory through the library."""
import numpy as np
import pytest

from paper_2605_23200_amd import diagnostics as D
from paper_2605_23200_amd import inputs


def test_region_wipeout_rate():
    present = np.arange(40)                       # regions of 10: 0..3
    assert D.region_wipeout_rate(present, np.array([0, 11, 25, 39]), 10) == 0.0
    assert D.region_wipeout_rate(present, np.array([0, 1, 2, 39]), 10) == 0.5
    assert D.region_wipeout_rate(present, np.array([], int), 10) == 1.0
    # regions that had no token before the event do not count
    assert D.region_wipeout_rate(np.array([3, 4, 95]), np.array([95]), 10) == 0.5


def test_span_wipeout():
    spans = np.array([[10, 20, 1.5], [30, 35, 1.5], [50, 60, 1.5], [90, 95, 1.5]])
    present = np.concatenate([np.arange(0, 40), np.arange(50, 60)])       # the last span was never in the cache
    assert D.span_wipeout(spans, present, np.array([0, 12, 55])) == (3, 1)  # [30, 35) lost
    assert D.span_wipeout(spans, present, present) == (3, 0)
    assert D.span_wipeout(spans, present, np.array([], int)) == (3, 3)
    assert D.span_wipeout(spans, np.array([20, 29, 35, 49]), np.array([20])) == (0, 0)   # stop is exclusive


def test_retained_iou():
    assert D.retained_iou(np.array([1, 2, 3]), np.array([1, 2, 3])) == 1.0
    assert D.retained_iou(np.array([1, 2, 3, 4]), np.array([3, 4, 5, 6])) == pytest.approx(2 / 6)
    assert D.retained_iou(np.array([1]), np.array([2])) == 0.0


def test_retention_profile_and_segment_stats():
    present = np.arange(100)
    prof = D.retention_profile(present, np.arange(0, 50), bins=4)
    np.testing.assert_allclose(prof, [1, 1, 0, 0])
    assert D.segment_stats(np.array([0, 10, 10, 40, 100, 100])) == (3, pytest.approx(100 / 3))


@pytest.mark.gpu
def test_trajectory_on_the_gpu():
    w = inputs.CONFIGS[0].scaled(H=2, T=2048, budget=512, n_append=128, S=8)
    recs = D.run_trajectory(w, n_events=3)
    assert len(recs) == 3
    for e, rec in enumerate(recs):
        for i in range(w.units):
            assert len(rec.kept[i]) == 512 and np.all(np.isin(rec.kept[i], rec.present[i]))
            assert np.all(np.diff(rec.present[i]) > 0) and np.all(np.diff(rec.kept[i]) > 0)
            # q_min = 1: every non-empty segment keeps something, so no segment is wiped out
            b = rec.bounds[i]
            for s in range(w.S):
                if b[s + 1] > b[s]:
                    seg_tokens = rec.present[i][b[s]:b[s + 1]]
                    assert np.isin(seg_tokens, rec.kept[i]).any()
        if e > 0:                                  # the cache of event e is what event e-1 kept plus the fresh tokens
            for i in range(w.units):
                assert np.array_equal(rec.present[i][:512], recs[e - 1].kept[i])
    sp = D.planted_spans(w)
    s_ams = D.summarize(recs, region=32, unit_spans=sp)
    recs_top = D.run_trajectory(w.scaled(S=1), n_events=3)
    s_top = D.summarize(recs_top, region=32, unit_spans=sp)
    print("AMS:", s_ams)
    print("global top-k:", s_top)
    for s in (s_ams, s_top):
        assert 0 <= s["region_wipeout_rate"] <= 1 and 0 <= s["retained_iou"] <= 1
        assert 0 <= s["span_wipeout_rate"] <= 1 and 0 <= s["spans_lost_at_end"] <= 1
    assert s_top["avg_segments"] == 1.0 and 1 <= s_ams["avg_segments"] <= 8
    # the same trajectories free-running through the CPU oracle (its own scores, its own selections): the kept
    # sets agree except where two scores are within rounding of each other, and the span figures agree
    from oracle import ams_oracle as O
    for ww, got in ((w, recs), (w.scaled(S=1), recs_top)):
        want = _oracle_trajectory(O, ww, 3)
        gone_g = gone_o = 0
        for e in range(3):
            for i in range(ww.units):
                assert D.retained_iou(got[e].kept[i], want[e].kept[i]) > 0.995
                gone_g += D.span_wipeout(sp[i], got[e].present[i], got[e].kept[i])[1]
                gone_o += D.span_wipeout(sp[i], want[e].present[i], want[e].kept[i])[1]
        assert abs(gone_g - gone_o) <= 1


def _oracle_trajectory(O, w, n_events):
    """run_trajectory through the CPU oracle (test infrastructure): same inputs, same bookkeeping."""
    host = inputs.dense_cache(w, n_threads=4)
    ids = inputs.unit_ids(w)
    K = {u: host["K"][l, b, h].copy() for u, (l, b, h) in enumerate(ids)}
    V = {u: host["V"][l, b, h].copy() for u, (l, b, h) in enumerate(ids)}
    credit = {u: np.zeros(w.T, np.float32) for u in range(w.units)}
    pos = {u: np.arange(w.T) for u in range(w.units)}
    next_id, out = w.T, []
    for e in range(n_events):
        rec = D.EventRecord()
        for u, (l, b, h) in enumerate(ids):
            Q = inputs.unit_q(w, l, b, h, e).reshape(-1, w.D)
            r = O.compress_unit(Q, K[u], V[u], credit[u], G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam, beta=w.beta,
                                eps=w.eps, q_min=w.q_min)
            idx = r["idx"]
            rec.present.append(pos[u].copy())
            rec.kept.append(pos[u][idx])
            rec.bounds.append(r["bounds"])
            fk, fv = inputs.unit_fresh_rows(w, l, b, h, e + 1, w.n_append)
            K[u] = np.concatenate([r["K_out"], fk])
            V[u] = np.concatenate([r["V_out"], fv])
            credit[u] = np.concatenate([r["credit_out"], np.zeros(w.n_append, np.float32)])
            pos[u] = np.concatenate([pos[u][idx], np.arange(next_id, next_id + w.n_append)])
        next_id += w.n_append
        out.append(rec)
    return out
