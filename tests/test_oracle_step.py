"""Whole-event invariants of the oracle on planted-span inputs, gather checks, generator checks."""
import numpy as np
import pytest

from paper_2605_23200_amd import inputs


def _small(**kw):
    base = inputs.CONFIGS[0].scaled(T=700, budget=128, S=8, n_spans=3, span_len=(16, 48), H=2)
    return base.scaled(**kw)


def _unit(w, h=0, T=None):
    T = T or w.T
    q = inputs.unit_q(w, 0, 0, h)
    k, v = inputs.unit_kv(w, 0, 0, h, T, q)
    return q, k, v


def test_step_invariants(oracle):
    w = _small()
    q, k, v = _unit(w)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam)
    assert r["n_kept"] == w.budget
    assert np.all(np.diff(r["idx"]) > 0) and r["idx"][0] >= 0 and r["idx"][-1] < w.T
    for i in range(w.S):
        a, b = r["bounds"][i], r["bounds"][i + 1]
        assert ((r["idx"] >= a) & (r["idx"] < b)).sum() == r["quota"][i]
        if b > a:
            assert r["quota"][i] >= 1                     # no region is wiped out
    np.testing.assert_array_equal(r["K_out"], k[r["idx"]])
    np.testing.assert_array_equal(r["V_out"], v[r["idx"]])
    np.testing.assert_array_equal(r["credit_out"], r["credit"][r["idx"]])
    # planted spans attract mass: the densest tenth of positions by mass overlaps the spans
    prof = inputs.span_shift_profile(w, 0, w.T)
    top = np.argsort(-r["m_used"])[: w.T // 10]
    assert (prof[top] > 0).mean() > 2 * (prof > 0).mean()


def test_budget_at_least_length_keeps_all(oracle):
    w = _small(T=90, budget=128)
    q, k, v = _unit(w)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam)
    assert r["n_kept"] == 90
    np.testing.assert_array_equal(r["idx"], np.arange(90))
    np.testing.assert_array_equal(r["K_out"], k)


def test_single_segment_equals_global_topk(oracle):
    w = _small(S=1)
    q, k, v = _unit(w)
    r = oracle.compress_unit(q, k, v, np.zeros(w.T, np.float32), G=w.G, W=w.W, budget=w.budget, S=1, lam=w.lam)
    order = np.argsort(-r["g"].astype(np.float64), kind="stable")
    np.testing.assert_array_equal(r["idx"], np.sort(order[: w.budget]))


def test_ema_zero_reproduces_raw_boundaries(oracle):
    w = _small()
    q, k, v = _unit(w)
    credit = np.random.default_rng(0).random(w.T).astype(np.float32)
    r0 = oracle.compress_unit(q, k, v, credit, G=w.G, W=w.W, budget=w.budget, S=w.S, lam=0.0)
    m = oracle.mass(r0["u"], w.eps)
    b, sm = oracle.segment(m, w.S)
    np.testing.assert_array_equal(r0["bounds"], b)
    np.testing.assert_array_equal(r0["m_used"], m)
    r9 = oracle.compress_unit(q, k, v, credit, G=w.G, W=w.W, budget=w.budget, S=w.S, lam=0.9)
    assert not np.array_equal(r9["bounds"], b)            # with history the boundaries move


def test_stage_chain_equals_whole_unit(oracle):
    w = _small(dtype="bf16", G=2, W=4)
    q, k, v = _unit(w)
    credit = np.random.default_rng(1).random(w.T).astype(np.float32) / w.T
    r = oracle.compress_unit(q, k, v, credit, G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam,
                             scorer=oracle.SCORER_EXPECTED)
    u, g = oracle.score(q.reshape(-1, w.D), k, w.G, w.W, oracle.SCORER_EXPECTED)
    m_used, c = oracle.ema(oracle.mass(u, w.eps), credit, w.lam, w.beta)
    bounds, sm = oracle.segment(m_used, w.S)
    quota = oracle.quota(bounds, sm, w.budget, w.q_min)
    idx = oracle.select(g, bounds, quota)
    Ko, Vo, co = oracle.compact(k, v, c, idx)
    for name, val in (("u", u), ("g", g), ("m_used", m_used), ("bounds", bounds), ("seg_mass", sm),
                      ("quota", quota), ("idx", idx), ("K_out", Ko), ("V_out", Vo), ("credit_out", co),
                      ("credit", c)):
        np.testing.assert_array_equal(r[name], val, err_msg=name)


def test_compress_many_matches_unit_calls(oracle):
    w = _small(H=3)
    Q = np.stack([inputs.as_f32(inputs.unit_q(w, 0, 0, h)).reshape(-1, w.D) for h in range(3)])
    KV = [_unit(w, h) for h in range(3)]
    K = np.stack([inputs.as_f32(x[1]) for x in KV])
    credit = np.zeros((3, w.T), np.float32)
    idx, n_kept, nthr = oracle.compress_many(Q, K, credit, G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam,
                                             n_threads=2)
    assert nthr == 2
    for h in range(3):
        r = oracle.compress_unit(KV[h][0], KV[h][1], KV[h][2], np.zeros(w.T, np.float32), G=w.G, W=w.W,
                                 budget=w.budget, S=w.S, lam=w.lam)
        np.testing.assert_array_equal(idx[h, : n_kept[h]], r["idx"])
        np.testing.assert_array_equal(credit[h], r["credit"])


def test_paged_gather_equals_dense_gather(oracle):
    # App. E: materialising head-wise selections into fresh paged blocks is the dense gather
    w = inputs.CONFIGS[2].scaled(L=1, B=3, H=2, T=200, T_min=50, n_spans=2, span_len=(8, 16))
    lens = inputs.seq_lens(w)
    dense = inputs.dense_cache(w, n_threads=2)
    kept = 40
    src, dst, n_slots = inputs.block_tables(w, lens, kept)
    Kp = inputs.paged_pool_from_dense(w, dense["K"], lens, src, n_slots)[0]
    Vp = inputs.paged_pool_from_dense(w, dense["V"], lens, src, n_slots)[0]
    Ko, Vo = Kp.copy(), Vp.copy()
    rng = np.random.default_rng(5)
    for b in range(w.B):
        for h in range(w.H):
            idx = np.sort(rng.choice(int(lens[b]), size=kept, replace=False)).astype(np.int32)
            oracle.compact_paged(Kp, Vp, src[b], Ko, Vo, dst[b], w.block, h, idx)
            Kd, Vd, _ = oracle.compact(dense["K"][0, b, h], dense["V"][0, b, h], np.zeros(w.T, np.float32), idx)
            j = np.arange(kept)
            slots = dst[b, j // w.block].astype(np.int64) * w.block + j % w.block
            np.testing.assert_array_equal(Ko[slots, h], Kd)
            np.testing.assert_array_equal(Vo[slots, h], Vd)
    # source blocks untouched
    used = np.concatenate([src[b, : (int(lens[b]) + 15) // 16] for b in range(w.B)])
    for blk in used:
        np.testing.assert_array_equal(Ko[blk * 16:(blk + 1) * 16], Kp[blk * 16:(blk + 1) * 16])


def test_generator_is_reproducible_and_unit_addressable():
    w = inputs.CONFIGS[1].scaled(L=2, H=2, T=512, n_spans=4, span_len=(16, 64))
    a = inputs.dense_cache(w, n_threads=2)
    b = inputs.dense_cache(w, n_threads=1)
    for k in ("Q", "K", "V"):
        np.testing.assert_array_equal(a[k], b[k])
    q = inputs.unit_q(w, 1, 0, 1)
    kk, vv = inputs.unit_kv(w, 1, 0, 1, w.T, q)
    np.testing.assert_array_equal(a["K"][1, 0, 1], kk)
    np.testing.assert_array_equal(a["Q"][1, 0, w.G:2 * w.G], q)
    assert a["K"].dtype == np.uint16
    kf = inputs.as_f32(a["K"][0, 0, 0])
    assert abs(kf.std() - 1.0) < 0.1


def test_trajectory_credit_carries_over(oracle):
    # four events with fresh tokens appended in between; credit of kept tokens is gathered, new ones start at 0
    w = _small()
    q, k, v = _unit(w)
    credit = np.zeros(w.T, np.float32)
    for e in range(3):
        r = oracle.compress_unit(q, k, v, credit, G=w.G, W=w.W, budget=w.budget, S=w.S, lam=w.lam)
        assert r["n_kept"] == w.budget
        fk, fv = inputs.unit_fresh_rows(w, 0, 0, 0, e + 1, 32)
        k = np.concatenate([r["K_out"], fk])
        v = np.concatenate([r["V_out"], fv])
        credit = np.concatenate([r["credit_out"], np.zeros(32, np.float32)])
        q = inputs.unit_q(w, 0, 0, 0, e + 1)
        assert credit[: w.budget].min() > 0
