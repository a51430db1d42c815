"""Pins for the causal window with padded observations (App. A "Mass construction")."""
import os

import numpy as np
from scipy.special import softmax

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example_causal.txt")


def _read(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = np.array([float(x) for x in v])
    return out


def test_worked_example(oracle):
    w = _read(GOLD)
    K = (w["ln2_multiples"] * np.log(2.0)).astype(np.float32).reshape(-1, 1)
    Q = np.ones((2, 1), np.float32)
    u, g = oracle.score(Q, K, 1, 2, causal=True)
    np.testing.assert_allclose(u, w["u_causal_num"] / w["u_causal_den"], rtol=2e-7)
    np.testing.assert_array_equal(g, u)
    u, _ = oracle.score(Q, K, 1, 2, causal=False)
    np.testing.assert_allclose(u, w["u_plain_num"] / w["u_plain_den"], rtol=2e-7)


def _masked_rows(Q, K, G, W):
    """Rows of causal attention from a library softmax over logits with -inf where a query cannot look."""
    T, D = K.shape
    logits = Q.astype(np.float64) @ K.astype(np.float64).T / np.sqrt(D)
    pos = T - W + np.tile(np.arange(W), G)                     # position of query n = (head, w)
    logits[np.arange(T)[None, :] > pos[:, None]] = -np.inf
    rows = np.zeros_like(logits)
    ok = pos >= 0
    rows[ok] = softmax(logits[ok], axis=1)
    return rows, pos


def test_window_of_one_query_is_not_changed(oracle):
    rng = np.random.default_rng(0)
    Q = rng.standard_normal((3, 16)).astype(np.float32)
    K = rng.standard_normal((50, 16)).astype(np.float32)
    a = oracle.score(Q, K, 3, 1, causal=True)
    b = oracle.score(Q, K, 3, 1, causal=False)
    np.testing.assert_array_equal(a[0], b[0])


def test_keys_older_than_the_window_get_the_plain_mean_of_masked_rows(oracle):
    rng = np.random.default_rng(1)
    G, W, T, D = 2, 6, 40, 8
    Q = rng.standard_normal((G * W, D)).astype(np.float32)
    K = rng.standard_normal((T, D)).astype(np.float32)
    u, _ = oracle.score(Q, K, G, W, causal=True)
    rows, _ = _masked_rows(Q, K, G, W)
    np.testing.assert_allclose(u[: T - W + 1], rows.mean(axis=0)[: T - W + 1], rtol=1e-6)
    # and they differ from the unmasked usage: the mask is really applied
    u_plain, _ = oracle.score(Q, K, G, W, causal=False)
    assert np.abs(u_plain[: T - W + 1] - u[: T - W + 1]).max() > 1e-4


def test_single_head_suffix_keys(oracle):
    # G = 1: key t of the suffix is seen by the T - t newest queries; the others count as the largest seen value
    rng = np.random.default_rng(2)
    W, T, D = 8, 30, 4
    Q = rng.standard_normal((W, D)).astype(np.float32)
    K = rng.standard_normal((T, D)).astype(np.float32)
    u, _ = oracle.score(Q, K, 1, W, causal=True)
    rows, pos = _masked_rows(Q, K, 1, W)
    for t in range(T - W + 1, T):
        seen = rows[pos >= t, t]
        assert len(seen) == T - t
        np.testing.assert_allclose(u[t], (seen.sum() + (W - len(seen)) * seen.max()) / W, rtol=1e-6)
    # the newest key has a single observation: its usage is that probability itself
    np.testing.assert_allclose(u[T - 1], rows[W - 1, T - 1], rtol=1e-6)


def test_identical_keys_closed_form(oracle):
    # all keys equal: a query that sees v keys gives each 1/v; padding takes the oldest seeing query's 1/(t+1)
    for (G, W, T) in ((2, 5, 12), (1, 4, 4), (3, 6, 3)):       # the last case has T < W: queries before position 0 do not exist
        K = np.ones((T, 4), np.float32)
        Q = np.random.default_rng(4).standard_normal((G * W, 4)).astype(np.float32)
        u, _ = oracle.score(Q, K, G, W, causal=True)
        want = np.zeros(T)
        for t in range(T):
            tot, seen = 0.0, 0
            for w in range(W):
                v = T - W + w + 1
                if v >= t + 1:
                    tot += 1.0 / v
                    seen += 1
            want[t] = (tot + (W - seen) / (t + 1.0)) / W
        np.testing.assert_allclose(u, want, rtol=1e-6)


def test_last_query_score_ignores_the_mask(oracle):
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((8, 8)).astype(np.float32)
    K = rng.standard_normal((25, 8)).astype(np.float32)
    _, g1 = oracle.score(Q, K, 2, 4, scorer=oracle.SCORER_LAST_QUERY, causal=True)
    _, g0 = oracle.score(Q, K, 2, 4, scorer=oracle.SCORER_LAST_QUERY, causal=False)
    np.testing.assert_array_equal(g1, g0)
