"""Pins of the redundancy-aware score of the oracle (amso_redundancy_score): a hand-worked example, closed
forms (identical keys, orthonormal keys, lambda = 0 and 1), the library softmax on numpy cosines, the linear
identity for the mean cosine, invariances."""
import os

import numpy as np
import pytest
from scipy.special import softmax

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example_redundancy.txt")


def _gold():
    vals = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array([float(x) for x in v])
    return vals


def test_worked_example(oracle):
    g0 = _gold()
    K = np.array([[1, 0], [0, 1], [3, 3]], np.float32)
    g = oracle.redundancy_score(g0["u"].astype(np.float32), K, mix_lambda=float(g0["lambda"][0]), kernel=1)
    np.testing.assert_allclose(g, g0["g"], rtol=0, atol=2e-8)


def test_identical_and_orthonormal_keys_give_a_uniform_penalty(oracle):
    rng = np.random.default_rng(0)
    u = rng.random(16).astype(np.float32)
    for K in (np.tile(rng.normal(size=(1, 32)), (16, 1)), np.eye(32)[:16] * 3.0):
        g = oracle.redundancy_score(u, K.astype(np.float32), mix_lambda=0.07, kernel=1)
        np.testing.assert_allclose(g, 0.07 * u.astype(np.float64) - 0.93 / 16, rtol=1e-6, atol=1e-9)


def test_against_library_softmax_of_numpy_cosines(oracle):
    rng = np.random.default_rng(1)
    T, D = 70, 24
    K = rng.normal(size=(T, D)).astype(np.float32)
    K[10:20] += 2.0                                    # a redundant cluster
    u = rng.random(T).astype(np.float32)
    Kn = K.astype(np.float64) / np.linalg.norm(K.astype(np.float64), axis=1, keepdims=True)
    cos = Kn @ Kn.T
    r = (cos.sum(1) - np.diag(cos)) / (T - 1)
    for kernel in (1, 7):
        a = u.astype(np.float64)
        if kernel > 1:
            a = oracle.pool(u, kernel).astype(np.float64)
        want = 0.07 * a - 0.93 * softmax(r)
        got = oracle.redundancy_score(u, K, mix_lambda=0.07, kernel=kernel)
        np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-9)
    # the cluster members are the most redundant: they get the largest penalty
    p = (0.07 * u - oracle.redundancy_score(u, K, mix_lambda=0.07, kernel=1)) / 0.93
    assert set(np.argsort(-p)[:10]) == set(range(10, 20))
    # linear identity: sum over s of cos(k_t, k_s) = khat_t . (sum of khat), minus the self term
    S = Kn.sum(0)
    np.testing.assert_allclose(r, (Kn @ S - 1.0) / (T - 1), rtol=1e-12, atol=1e-14)


def test_limits_of_the_mixing_weight_and_edge_cases(oracle):
    rng = np.random.default_rng(2)
    K = rng.normal(size=(40, 8)).astype(np.float32)
    u = rng.random(40).astype(np.float32)
    np.testing.assert_array_equal(oracle.redundancy_score(u, K, mix_lambda=1.0, kernel=1), u)
    g0 = oracle.redundancy_score(u, K, mix_lambda=0.0, kernel=1)
    assert np.all(g0 < 0) and abs(g0.astype(np.float64).sum() + 1.0) < 1e-6      # minus a distribution
    one = oracle.redundancy_score(np.array([0.4], np.float32), K[:1], mix_lambda=0.3, kernel=1)
    np.testing.assert_allclose(one, [0.3 * np.float32(0.4) - 0.7], rtol=1e-6)        # a single key: p = 1
    Kz = K.copy()
    Kz[5] = 0.0                                        # a zero key: cosine 0 to everything, no NaN
    assert np.isfinite(oracle.redundancy_score(u, Kz, mix_lambda=0.07, kernel=1)).all()


def test_invariances(oracle):
    rng = np.random.default_rng(3)
    K = rng.normal(size=(50, 16)).astype(np.float32)
    u = rng.random(50).astype(np.float32)
    g = oracle.redundancy_score(u, K, mix_lambda=0.07, kernel=1)
    perm = rng.permutation(50)
    np.testing.assert_allclose(oracle.redundancy_score(u[perm], K[perm], mix_lambda=0.07, kernel=1), g[perm],
                               rtol=1e-6, atol=1e-9)
    scale = (2.0 ** rng.integers(-3, 4, size=50)).astype(np.float32)[:, None]     # exact rescaling of each key
    np.testing.assert_allclose(oracle.redundancy_score(u, K * scale, mix_lambda=0.07, kernel=1), g, rtol=1e-6, atol=1e-9)
    with pytest.raises(RuntimeError):
        oracle.redundancy_score(u, K, mix_lambda=1.5, kernel=1)
    with pytest.raises(RuntimeError):
        oracle.redundancy_score(u, K, mix_lambda=0.1, kernel=4)


def test_whole_event_uses_the_stage(oracle):
    from paper_2605_23200_amd import inputs
    w = inputs.CONFIGS[0].scaled(H=1, T=300, budget=64, S=4, n_spans=2, span_len=(8, 30))
    host = inputs.dense_cache(w, n_threads=1)
    Q, K, V = host["Q"][0, 0, 0:w.G].reshape(-1, w.D), host["K"][0, 0, 0], host["V"][0, 0, 0]
    r = oracle.compress_unit(Q, K, V, np.zeros(w.T, np.float32), G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam,
                             scorer=oracle.SCORER_REDUNDANCY, mix_lambda=0.1, score_kernel=5)
    u, _ = oracle.score(Q, K, w.G, w.W, oracle.SCORER_MEAN_WINDOW)
    np.testing.assert_array_equal(r["u"], u)
    np.testing.assert_array_equal(r["g"], oracle.redundancy_score(u, K, mix_lambda=0.1, kernel=5))
    quota = oracle.quota(r["bounds"], r["seg_mass"], w.budget, 1)
    np.testing.assert_array_equal(r["idx"], oracle.select(r["g"], r["bounds"], quota))
