"""Pins for the oracle's usage / base-score stage (Sec. 3.2; Alg. 1 step 1; Sec. 3.3 plug-in scorer).

Nothing here calls the GPU.  The oracle is compared with an independent library softmax, with closed
forms and with algebraic identities that take a different route from the oracle's own code.
"""
import numpy as np
import pytest
from scipy.special import softmax


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def test_usage_is_column_mean_of_library_softmax(oracle):
    G, W, T, D = 3, 5, 37, 16
    Q, K = _rand(1, G * W, D), _rand(2, T, D)
    u, g = oracle.score(Q, K, G, W, oracle.SCORER_MEAN_WINDOW)
    p = softmax(Q.astype(np.float64) @ K.astype(np.float64).T / np.sqrt(D), axis=1)   # [N, T]
    np.testing.assert_allclose(u, p.mean(axis=0), rtol=2e-7, atol=0)
    np.testing.assert_array_equal(u, g)
    assert abs(float(u.astype(np.float64).sum()) - 1.0) < 1e-6


def test_scale_is_inverse_sqrt_head_dim(oracle):
    # one query, two keys: p = softmax([a, 0]) with a = q.k0/sqrt(D); closed form logistic
    D = 4
    Q = np.array([[1, 2, 3, 4]], np.float32)
    K = np.array([[0.5, 0.5, 0.5, 0.5], [0, 0, 0, 0]], np.float32)
    u, _ = oracle.score(Q, K, 1, 1)
    a = 5.0 / 2.0
    np.testing.assert_allclose(u, [1 / (1 + np.exp(-a)), 1 / (1 + np.exp(a))], rtol=2e-7)


def test_large_logits_do_not_overflow(oracle):
    D = 2
    Q = np.array([[300.0, 0.0]], np.float32)
    K = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 5.0]], np.float32)
    u, _ = oracle.score(Q, K, 1, 1)
    np.testing.assert_allclose(u, [0.5, 0.0, 0.5], atol=1e-30)


def test_last_query_scorer_uses_newest_query_of_each_head(oracle):
    G, W, T, D = 2, 3, 29, 8
    Q, K = _rand(3, G * W, D), _rand(4, T, D)
    u, g = oracle.score(Q, K, G, W, oracle.SCORER_LAST_QUERY)
    p = softmax(Q.astype(np.float64) @ K.astype(np.float64).T / np.sqrt(D), axis=1)
    newest = [h * W + (W - 1) for h in range(G)]          # query index n = head * W + window position
    np.testing.assert_allclose(g, p[newest].mean(axis=0), rtol=2e-7)
    np.testing.assert_allclose(u, p.mean(axis=0), rtol=2e-7)


def test_single_query_last_equals_mean(oracle):
    Q, K = _rand(5, 1, 8), _rand(6, 19, 8)
    u, g = oracle.score(Q, K, 1, 1, oracle.SCORER_LAST_QUERY)
    np.testing.assert_array_equal(u, g)


def test_keydiff_closed_forms(oracle):
    Q = _rand(7, 2, 4)
    v = np.array([1.0, 2.0, -1.0, 0.5], np.float32)
    # every key a positive multiple of v -> mean key parallel to v -> cosine 1 -> score -1
    K = np.stack([v * a for a in (0.5, 1.0, 3.0, 8.0)])
    _, g = oracle.score(Q, K, 1, 2, oracle.SCORER_KEYDIFF)
    np.testing.assert_allclose(g, -1.0, rtol=1e-6)
    # keys e1, e2: mean (e1+e2)/2, cosine 1/sqrt(2) for both
    K = np.eye(4, dtype=np.float32)[:2]
    _, g = oracle.score(Q, K, 1, 2, oracle.SCORER_KEYDIFF)
    np.testing.assert_allclose(g, -1 / np.sqrt(2), rtol=1e-6)
    # 3*e1, -e1, e2 : mean (2/3, 1/3, 0, 0); cos = 2/sqrt5, -2/sqrt5, 1/sqrt5
    K = np.array([[3, 0, 0, 0], [-1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
    _, g = oracle.score(Q, K, 1, 2, oracle.SCORER_KEYDIFF)
    np.testing.assert_allclose(g, [-2 / np.sqrt(5), 2 / np.sqrt(5), -1 / np.sqrt(5)], rtol=1e-6)
    assert np.all(np.abs(g) <= 1 + 1e-6)


def test_keydiff_permutation_equivariant(oracle):
    Q, K = _rand(8, 4, 8), _rand(9, 33, 8)
    perm = np.random.default_rng(0).permutation(33)
    _, g = oracle.score(Q, K, 2, 2, oracle.SCORER_KEYDIFF)
    _, gp = oracle.score(Q, K[perm], 2, 2, oracle.SCORER_KEYDIFF)
    np.testing.assert_allclose(gp, g[perm], rtol=1e-6, atol=1e-7)


def test_expected_attention_equals_mean_plus_half_variance_of_logits(oracle):
    # k' Sigma k = Var_n(q_n.k) and mu.k = mean_n(q_n.k): the oracle goes through the explicit
    # D x D covariance, this check through the per-query logits.
    G, W, T, D = 2, 6, 41, 16
    Q, K = _rand(10, G * W, D), _rand(11, T, D)
    _, g = oracle.score(Q, K, G, W, oracle.SCORER_EXPECTED)
    s = Q.astype(np.float64) @ K.astype(np.float64).T / np.sqrt(D)        # [N, T]
    np.testing.assert_allclose(g, s.mean(axis=0) + 0.5 * s.var(axis=0), rtol=1e-6, atol=1e-7)


def test_expected_attention_identical_queries_give_the_logit(oracle):
    q = _rand(12, 1, 8)
    Q = np.repeat(q, 5, axis=0)
    K = _rand(13, 17, 8)
    _, g = oracle.score(Q, K, 1, 5, oracle.SCORER_EXPECTED)
    np.testing.assert_allclose(g, (q.astype(np.float64) @ K.astype(np.float64).T / np.sqrt(8))[0],
                               rtol=1e-6, atol=1e-7)


def test_expected_attention_is_log_gaussian_moment(oracle):
    # Monte-Carlo check of the closed form log E[exp(q.k/sqrt(D))], q ~ N(mu, Sigma) fitted to the window
    G, W, D = 1, 64, 3
    Q = (0.3 * _rand(14, W, D)).astype(np.float32)
    K = _rand(15, 4, D)
    _, g = oracle.score(Q, K, G, W, oracle.SCORER_EXPECTED)
    mu = Q.astype(np.float64).mean(axis=0)
    cov = np.cov(Q.astype(np.float64).T, bias=True)
    draws = np.random.default_rng(16).multivariate_normal(mu, cov, size=400000)
    mc = np.log(np.exp(draws @ K.astype(np.float64).T / np.sqrt(D)).mean(axis=0))
    np.testing.assert_allclose(g, mc, atol=5e-3)


def test_bf16_inputs_are_widened_exactly(oracle):
    from paper_2605_23200_amd import inputs
    Q, K = _rand(17, 4, 8), _rand(18, 21, 8)
    Qb, Kb = inputs.to_bf16_bits(Q), inputs.to_bf16_bits(K)
    u1, _ = oracle.score(Qb, Kb, 2, 2)
    u2, _ = oracle.score(inputs.bf16_bits_to_f32(Qb), inputs.bf16_bits_to_f32(Kb), 2, 2)
    np.testing.assert_array_equal(u1, u2)
    # round-to-nearest-even: 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0)
    assert inputs.bf16_bits_to_f32(inputs.to_bf16_bits(np.array([1 + 2.0 ** -8], np.float32)))[0] == 1.0
    assert inputs.bf16_bits_to_f32(inputs.to_bf16_bits(np.array([1 + 3 * 2.0 ** -8], np.float32)))[0] == 1 + 2.0 ** -6


# --- value-weighted expected attention (Sec. 3.3 plug-in scorer; the paper gives the scorer's epsilon 1e-2) ---

def test_value_weight_closed_forms(oracle):
    # equal scores: p = 1/T; rows (3,4,0..) and (0,..,0,12,5) have lengths 5 and 13
    T, D = 4, 8
    V = np.zeros((T, D), np.float32)
    V[0, :2] = (3, 4)
    V[1, -2:] = (12, 5)
    V[2, 0] = 1
    g = oracle.value_weight(np.full(T, 7.0, np.float32), V, eps=0.25)
    np.testing.assert_allclose(g, [0.5 * 5, 0.5 * 13, 0.5 * 1, 0.0], rtol=1e-7)
    # eps = 0 and unit values: the softmax of the scores itself, here ln 1, ln 2, ln 5 -> 1/8, 2/8, 5/8
    V = np.zeros((3, 4), np.float32)
    V[:, 1] = 1
    g = oracle.value_weight(np.log(np.array([1, 2, 5], np.float32)), V, eps=0.0)
    np.testing.assert_allclose(g, [0.125, 0.25, 0.625], rtol=1e-6)


def test_value_weight_against_library_routines(oracle):
    from scipy.special import softmax
    rng = np.random.default_rng(8)
    T, D = 500, 128
    e = (rng.standard_normal(T) * 4).astype(np.float32)
    e[17] = 60.0                                   # a dominant token: no overflow, p close to 1
    V = rng.standard_normal((T, D)).astype(np.float32)
    g = oracle.value_weight(e, V, eps=1e-2)
    want = (softmax(e.astype(np.float64)) + 1e-2) * np.linalg.norm(V.astype(np.float64), axis=1)
    np.testing.assert_allclose(g, want, rtol=1e-6)
    assert np.argmax(g) == 17
    # bf16 values are widened exactly
    from paper_2605_23200_amd import inputs
    Vb = inputs.to_bf16_bits(V)
    g2 = oracle.value_weight(e, Vb, eps=1e-2)
    want2 = (softmax(e.astype(np.float64)) + 1e-2) * np.linalg.norm(inputs.bf16_bits_to_f32(Vb).astype(np.float64), axis=1)
    np.testing.assert_allclose(g2, want2, rtol=1e-6)


def test_whole_event_with_value_weighted_scorer(oracle):
    from paper_2605_23200_amd import inputs
    w = inputs.CONFIGS[0].scaled(T=600, budget=96, S=8, n_spans=3, span_len=(16, 48), H=1)
    q = inputs.unit_q(w, 0, 0, 0)
    k, v = inputs.unit_kv(w, 0, 0, 0, w.T, q)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam,
                             scorer=oracle.SCORER_EXPECTED_VNORM)
    u, e = oracle.score(q, k, w.G, w.W, oracle.SCORER_EXPECTED)
    np.testing.assert_array_equal(r["u"], u)
    np.testing.assert_array_equal(r["g"], oracle.value_weight(e, v, 1e-2))
    np.testing.assert_array_equal(r["idx"], oracle.select(r["g"], r["bounds"], r["quota"]))
