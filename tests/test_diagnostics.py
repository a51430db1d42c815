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
    s_ams = D.summarize(recs, region=32)
    s_top = D.summarize(D.run_trajectory(w.scaled(S=1), n_events=3), region=32)
    print("AMS:", s_ams)
    print("global top-k:", s_top)
    for s in (s_ams, s_top):
        assert 0 <= s["region_wipeout_rate"] <= 1 and 0 <= s["retained_iou"] <= 1
    assert s_top["avg_segments"] == 1.0 and 1 <= s_ams["avg_segments"] <= 8
