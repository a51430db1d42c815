"""End-to-end parity of the fused compression step against the CPU oracle, through the C ABI.

Protocol: the scores and the mass the GPU produced are compared with the oracle's within relative
1e-5; every later stage of the oracle is then fed the GPU's own floats, so that quotas, kept
indices and gathered K/V bytes must agree exactly (selection "on identical score inputs").
"""
import numpy as np
import pytest
import torch

from paper_2605_23200_amd import binding as B
from paper_2605_23200_amd import inputs
from paper_2605_23200_amd.harness import Job
from gpu_util import assert_close_rel, assert_close_terms, score_term_magnitudes, to_dev, to_host, unit_list

pytestmark = pytest.mark.gpu


def _kv_out_host(job, host_dtype):
    """[units, keep, D] arrays of the compacted K, V."""
    w = job.w
    if not job.paged:
        return (to_host(job.Kd, host_dtype).reshape(job.units, job.keep, w.D),
                to_host(job.Vd, host_dtype).reshape(job.units, job.keep, w.D))
    Kp, Vp = to_host(job.K, host_dtype), to_host(job.V, host_dtype)
    Ko = np.zeros((job.units, job.keep, w.D), Kp.dtype)
    Vo = np.zeros_like(Ko)
    j = np.arange(job.keep)
    for i, (l, b, h) in enumerate(unit_list(w)):
        slots = job.dst_table_h[b, j // 16].astype(np.int64) * 16 + j % 16
        Ko[i], Vo[i] = Kp[l, slots, h], Vp[l, slots, h]
    return Ko, Vo


def check_units(oracle, job, host, credit_before, units, scorer=B.SCORER_MEAN_WINDOW, check_scores=True,
                unit_rows=None):
    """Full per-unit comparison of one finished step for the listed unit numbers.  unit_rows (optional):
    i -> (Q[N, D], K[T, D], V[T, D], K'[keep, D], V'[keep, D]) for jobs that have no host copy of the cache."""
    w = job.w
    inter = job.intermediates()
    ids = unit_list(w)
    sel = torch.tensor(units, device=job.device)
    u_g, g_g, m_g = (to_host(x[sel]) for x in (inter.u, inter.g, inter.m_used))
    b_g, sm_g, q_g = (to_host(x[sel]) for x in (inter.bounds, inter.seg_mass, inter.quota))
    idx_g, nk_g = to_host(job.idx[sel]), to_host(job.n_kept[sel])
    cred_g, cdst_g = to_host(job.credit[sel]), to_host(job.credit_dst[sel])
    if unit_rows is None:
        Ko, Vo = _kv_out_host(job, host["K"].dtype)
    lens = host["seq_lens"]

    def one(j, i):
        l, b, h = ids[i]
        T = int(lens[b])
        if unit_rows is None:
            Qh = host["Q"][l, b, h * w.G:(h + 1) * w.G].reshape(-1, w.D)
            Kh, Vh = host["K"][l, b, h, :T], host["V"][l, b, h, :T]
            Ko_i, Vo_i = Ko[i], Vo[i]
        else:
            Qh, Kh, Vh, Ko_i, Vo_i = unit_rows(i)
        if check_scores:
            vnorm = scorer == B.SCORER_EXPECTED_VNORM
            uo, go = oracle.score(Qh, Kh, w.G, w.W,
                                  B.SCORER_EXPECTED if vnorm else (B.SCORER_MEAN_WINDOW if scorer == B.SCORER_REDUNDANCY
                                                                   else scorer), causal=w.causal)
            if vnorm:
                go = oracle.value_weight(go, Vh, 1e-2)
            assert_close_rel(u_g[j, :T], uo, what=f"u unit {i}")
            if scorer == B.SCORER_REDUNDANCY:       # the oracle's O(T^2) definition on the GPU's own usage
                go = oracle.redundancy_score(u_g[j, :T], Kh, mix_lambda=job.p.mix_lambda, kernel=job.p.score_kernel)
                a = (oracle.pool(u_g[j, :T], job.p.score_kernel) if job.p.score_kernel > 1 else u_g[j, :T]).astype(np.float64)
                mag = job.p.mix_lambda * np.abs(a) + np.abs(job.p.mix_lambda * a - go.astype(np.float64))
                assert_close_terms(g_g[j, :T], go, mag, what=f"g unit {i}")
            elif scorer in (B.SCORER_MEAN_WINDOW, B.SCORER_LAST_QUERY, B.SCORER_EXPECTED_VNORM):
                assert_close_rel(g_g[j, :T], go, what=f"g unit {i}")
            else:
                assert_close_terms(g_g[j, :T], go, score_term_magnitudes(scorer, Qh, Kh), what=f"g unit {i}")
        u_mass = oracle.pool(u_g[j, :T], w.pool_kernel) if w.pool_kernel > 1 else u_g[j, :T]
        m_o, c_o = oracle.ema(oracle.mass(u_mass, w.eps), credit_before[i, :T], w.lam, w.beta)
        assert_close_rel(m_g[j, :T], m_o, what=f"m_used unit {i}")
        assert_close_rel(cred_g[j, :T], c_o, what=f"credit unit {i}")
        if w.seg_delta > 0:
            b_o, sm_o, _ = oracle.segment_adaptive(m_g[j, :T], w.seg_delta, w.l_min, w.l_max, w.S)
        else:
            b_o, sm_o = oracle.segment(m_g[j, :T], w.S)
        np.testing.assert_array_equal(b_g[j], b_o, err_msg=f"bounds unit {i}")
        assert_close_rel(sm_g[j], sm_o, what=f"seg_mass unit {i}")
        sinks, last, seg_budget = oracle.must_keep(T, w.budget, w.n_sink, w.n_last)
        q_o = oracle.quota(b_g[j], sm_g[j], seg_budget, w.q_min)
        np.testing.assert_array_equal(q_g[j], q_o, err_msg=f"quota unit {i}")
        n = min(w.budget, T)
        i_o = oracle.finalize(g_g[j, :T], oracle.select(g_g[j, :T], b_g[j], q_g[j]), sinks, last, n)
        assert nk_g[j] == n == len(i_o)
        np.testing.assert_array_equal(idx_g[j, :n], i_o, err_msg=f"idx unit {i}")
        assert (idx_g[j, n:] == -1).all()
        np.testing.assert_array_equal(Ko_i[:n], Kh[i_o], err_msg=f"K' unit {i}")
        np.testing.assert_array_equal(Vo_i[:n], Vh[i_o], err_msg=f"V' unit {i}")
        np.testing.assert_array_equal(cdst_g[j, :n], cred_g[j, i_o], err_msg=f"credit' unit {i}")

    if len(units) <= 4:
        for j, i in enumerate(units):
            one(j, i)
    else:       # the oracle's C calls release the interpreter lock: units are checked side by side
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=16) as ex:
            for f in [ex.submit(one, j, i) for j, i in enumerate(units)]:
                f.result()


def check_properties_all_units(job):
    """Size-independent properties over every unit, evaluated on the device."""
    w, inter = job.w, job.intermediates()
    lens = job.lens.long().repeat_interleave(w.H).repeat(w.L)              # [units]
    keep = torch.minimum(lens, torch.tensor(w.budget, device=job.device))
    assert torch.equal(job.n_kept.long(), keep)
    idx = job.idx.long()
    col = torch.arange(w.budget, device=job.device)[None, :]
    valid = col < keep[:, None]
    assert bool(((idx >= 0) & (idx < lens[:, None]))[valid].all())
    assert bool((idx[~valid] == -1).all())
    inc = (idx[:, 1:] > idx[:, :-1]) | ~valid[:, 1:]
    assert bool(inc.all())                                                  # strictly ascending
    sinks = torch.clamp(keep, max=w.n_sink)
    last = torch.minimum(keep - sinks, torch.tensor(w.n_last, device=job.device))
    assert bool((inter.quota.long().sum(1) == keep - sinks - last).all())
    seg_of = torch.searchsorted(inter.bounds[:, 1:].contiguous().long(), idx.clamp(min=0), right=True)
    for s in range(w.S):                                                    # every segment holds its quota
        held = ((seg_of == s) & valid).sum(1)
        if w.n_sink or w.n_last:                                            # must-keep and backfill only add
            assert bool((held >= inter.quota[:, s].long()).all())
        else:
            assert torch.equal(held, inter.quota[:, s].long())
    if w.n_sink or w.n_last:                                                # the must-keep positions are in
        kept_mask = torch.zeros((job.units, job.t_stride + 1), dtype=torch.bool, device=job.device)
        kept_mask.scatter_(1, torch.where(valid, idx, torch.tensor(job.t_stride, device=job.device)), True)
        pos = torch.arange(job.t_stride, device=job.device)[None, :]
        must = (pos < sinks[:, None]) | ((pos >= (lens - last)[:, None]) & (pos < lens[:, None]))
        assert bool((kept_mask[:, :-1] | ~must).all())
    T = job.t_max
    tmask = torch.arange(job.t_stride, device=job.device)[None, :] < lens[:, None]
    usum = (inter.u.double() * tmask).sum(1)
    if w.causal:                                                            # padded observations only add
        assert float(usum.min()) > 1 - 1e-4 and float(usum.max()) < 1 + w.W
    else:
        assert float((usum - 1).abs().max()) < 1e-4                         # usage is a distribution
    msum = (inter.m_used.double() * tmask).sum(1)
    assert float((msum - 1).abs().max()) < 1e-5
    if not job.paged:                                                       # K' = K[idx], V' = V[idx] everywhere
        K = job.K.reshape(job.units, -1, w.D)
        V = job.V.reshape(job.units, -1, w.D)
        gi = idx.clamp(min=0)[:, :job.keep, None].expand(-1, -1, w.D)
        vmask = valid[:, :job.keep, None]
        assert bool(((torch.gather(K, 1, gi) == job.Kd.reshape(job.units, job.keep, w.D)) | ~vmask).all())
        assert bool(((torch.gather(V, 1, gi) == job.Vd.reshape(job.units, job.keep, w.D)) | ~vmask).all())


def test_config0_trajectory(oracle):
    """Config 0 as stated: fp32, 8 units, T = 4096, budget 1024, S = 8, four events, 256 fresh tokens between."""
    w = inputs.CONFIGS[0]
    host = inputs.dense_cache(w, n_threads=8)
    ids = unit_list(w)
    credit = np.zeros((w.units, w.T), np.float32)
    # the oracle's own free-running trajectory, for the divergence report
    free = [dict(K=host["K"][u], V=host["V"][u], c=np.zeros(w.T, np.float32)) for u in ids]
    agree = []
    for e in range(w.n_events):
        job = Job(w, host, credit=credit)
        job.step()
        torch.cuda.synchronize()
        check_units(oracle, job, host, credit, list(range(w.units)))
        check_properties_all_units(job)
        idx_g = to_host(job.idx)
        same = 0
        for i, (l, b, h) in enumerate(ids):
            f = free[i]
            r = oracle.compress_unit(host["Q"][l, b, h * w.G:(h + 1) * w.G], f["K"], f["V"], f["c"], G=w.G, W=w.W,
                                     budget=w.budget, S=w.S, lam=w.lam, beta=w.beta, eps=w.eps, q_min=w.q_min)
            same += int(np.array_equal(r["idx"], idx_g[i, :r["n_kept"]]))
            fk, fv = inputs.unit_fresh_rows(w, l, b, h, e + 1, w.n_append)
            f["K"], f["V"] = np.concatenate([r["K_out"], fk]), np.concatenate([r["V_out"], fv])
            f["c"] = np.concatenate([r["credit_out"], np.zeros(w.n_append, np.float32)])
        agree.append(same)
        # next event: kept rows + fresh rows, credit of kept rows carried, fresh Q window
        Ko, Vo = _kv_out_host(job, host["K"].dtype)
        cd = to_host(job.credit_dst)
        T_new = w.budget + w.n_append
        K2 = np.zeros((w.L, w.B, w.H, T_new, w.D), host["K"].dtype)
        V2 = np.zeros_like(K2)
        credit = np.zeros((w.units, T_new), np.float32)
        Q2 = np.zeros_like(host["Q"])
        for i, (l, b, h) in enumerate(ids):
            fk, fv = inputs.unit_fresh_rows(w, l, b, h, e + 1, w.n_append)
            K2[l, b, h] = np.concatenate([Ko[i], fk])
            V2[l, b, h] = np.concatenate([Vo[i], fv])
            credit[i, :w.budget] = cd[i]
            Q2[l, b, h * w.G:(h + 1) * w.G] = inputs.unit_q(w, l, b, h, e + 1)
        host = dict(Q=Q2, K=K2, V=V2, seq_lens=np.full(w.B, T_new, np.int32))
        w = w.scaled(T=T_new)
    print("free-running oracle vs GPU: units with identical kept sets per event:", agree)
    assert agree[0] >= 7          # first event: same inputs, only fp32-vs-fp64 rounding can flip a choice


def test_config1_literal_trajectory(oracle):
    """Config 1's trajectory as stated (first event at T = 32768 -> 2048, later events at 2048 + 128 appended
    tokens), on two layers: every event against the oracle, credit carried through the compaction."""
    w = inputs.CONFIGS[1].scaled(L=2)
    host = inputs.dense_cache(w, n_threads=16)
    ids = unit_list(w)
    credit = np.zeros((w.units, w.T), np.float32)
    for e in range(3):
        job = Job(w, host, credit=credit)
        job.step()
        torch.cuda.synchronize()
        check_properties_all_units(job)
        check_units(oracle, job, host, credit, [0, 5, w.units - 1] if e == 0 else list(range(w.units)))
        Ko, Vo = _kv_out_host(job, host["K"].dtype)
        cd = to_host(job.credit_dst)
        T_new = w.budget + w.n_append
        K2 = np.zeros((w.L, w.B, w.H, T_new, w.D), host["K"].dtype)
        V2 = np.zeros_like(K2)
        credit = np.zeros((w.units, T_new), np.float32)
        Q2 = np.zeros_like(host["Q"])
        for i, (l, b, h) in enumerate(ids):
            fk, fv = inputs.unit_fresh_rows(w, l, b, h, e + 1, w.n_append)
            K2[l, b, h] = np.concatenate([Ko[i], fk])
            V2[l, b, h] = np.concatenate([Vo[i], fv])
            credit[i, :w.budget] = cd[i]
            Q2[l, b, h * w.G:(h + 1) * w.G] = inputs.unit_q(w, l, b, h, e + 1)
        host = dict(Q=Q2, K=K2, V=V2, seq_lens=np.full(w.B, T_new, np.int32))
        w = w.scaled(T=T_new)
        assert credit.max() > 0                         # the carried credit is what the next event's EMA starts from


@pytest.fixture(scope="module")
def cfg1_job():
    w = inputs.CONFIGS[1]
    host = inputs.dense_cache(w, n_threads=16)
    job = Job(w, host)
    return w, host, job


def test_config1_full_size(oracle, cfg1_job):
    """Config 1 at full size in the launch configuration bench.py times: properties AND element-by-element
    parity against the oracle on all 256 units, two events so that the credit path does real work."""
    w, host, job = cfg1_job
    zeros = np.zeros((w.units, w.T), np.float32)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    every = list(range(w.units))
    check_units(oracle, job, host, zeros, every)
    credit1 = to_host(job.credit)[:, :w.T].copy()
    job.step()                                   # second event on the same cache: credit is now non-trivial
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, credit1, every, check_scores=False)


def test_config1_full_size_one_read(oracle, cfg1_job):
    """The same workload through the pinned one-read scorer (64 workgroups per unit, 32 units per cluster):
    usage of all 256 units against the oracle, the rest of the event on a sample."""
    w, host, _ = cfg1_job
    job = Job(w, host, score_path=B.SCORE_PATH_ONE_READ)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)))


def test_config1_full_size_paper_options(oracle, cfg1_job):
    """Config 1 at full size with everything the paper's default configuration switches on: target mass
    0.1 with L_min 16 / L_max 256, pooled usage, 4 sinks + 32 recent tokens, causal window."""
    w0, host, _ = cfg1_job
    cap = 10 + 1 + w0.T // 256
    w = w0.scaled(S=cap, seg_delta=0.1, l_min=16, l_max=256, pool_kernel=5, n_sink=4, n_last=32, causal=True)
    job = Job(w, host)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), [3, 200])
    n_seg = (job.intermediates().bounds[:, 1:] > job.intermediates().bounds[:, :-1]).sum(1)
    print("segments per unit: min", int(n_seg.min()), "max", int(n_seg.max()))
    assert int(n_seg.min()) >= 10 and int(n_seg.max()) <= cap


def test_config1_deterministic(cfg1_job):
    w, host, job = cfg1_job
    job.credit.zero_()
    job.step()
    a = (job.idx.clone(), job.Kd.clone(), job.intermediates().u.clone())
    job.credit.zero_()
    job.step()
    torch.cuda.synchronize()
    assert torch.equal(a[0], job.idx) and torch.equal(a[1], job.Kd) and torch.equal(a[2], job.intermediates().u)


def test_config2_paged_ragged(oracle):
    """Config 2 shapes on one layer: batch 64, ragged lengths 4096..16384, paged layout with permuted
    block tables, compaction into fresh blocks of the same pool."""
    w = inputs.CONFIGS[2].scaled(L=1)
    host = inputs.dense_cache(w, n_threads=16)
    job = Job(w, host)
    assert job.paged
    zeros = np.zeros((w.units, job.t_max), np.float32)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    lens = host["seq_lens"]
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    check_units(oracle, job, host, zeros, [shortest * w.H, longest * w.H + 3, 17 * w.H + 5, w.units - 1])
    # source blocks are untouched by the compaction
    Kp = to_host(job.K, np.uint16)
    for b in (shortest, longest):
        T = int(lens[b])
        p = np.arange(T)
        slots = job.src_table_h[b, p // 16].astype(np.int64) * 16 + p % 16
        np.testing.assert_array_equal(Kp[0, slots].transpose(1, 0, 2), host["K"][0, b, :, :T])


def test_config2_full_size(oracle):
    """Config 2 at full size (32 layers x 64 sequences x 8 KV heads = 16384 ragged units in the paged layout,
    about 95 GB on the device), the launch shapes `bench.py --config 2` times.  The values are drawn on the
    device, so the rows of the sampled units are read back through the block tables for the oracle."""
    from paper_2605_23200_amd.harness import DeviceFilledPagedJob
    w = inputs.CONFIGS[2]
    job = DeviceFilledPagedJob(w)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    lens = job.lens_h
    ids = unit_list(w)
    src_t, dst_t = job.src_table.long(), job.dst_table.long()

    def rows(i):
        l, b, h = ids[i]
        T = int(lens[b])
        p = torch.arange(T, device=job.device)
        slots = src_t[b, p // 16] * 16 + p % 16
        j = torch.arange(job.keep, device=job.device)
        dslots = dst_t[b, j // 16] * 16 + j % 16
        Q = to_host(job.Q[l, b, h * w.G:(h + 1) * w.G].reshape(-1, w.D).view(torch.int16), np.uint16)
        return (Q, to_host(job.K[l, slots, h].view(torch.int16), np.uint16),
                to_host(job.V[l, slots, h].view(torch.int16), np.uint16),
                to_host(job.K[l, dslots, h].view(torch.int16), np.uint16),
                to_host(job.V[l, dslots, h].view(torch.int16), np.uint16))

    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    sample = [shortest * w.H + 1, 9 * w.B * w.H + longest * w.H + 6, w.units - 1]
    class ZeroCredit:  # credit_before[i, :T] without a [units, T] array of zeros
        def __getitem__(self, key):
            return np.zeros(job.t_max, np.float32)[key[1]]

    check_units(oracle, job, {"seq_lens": lens}, ZeroCredit(), sample, unit_rows=rows)


def test_config3_long_context(oracle):
    """Config 3 shapes on one layer and two heads: T = 131072, N = 7 x 32 = 224 queries, S = 32."""
    w = inputs.CONFIGS[3].scaled(L=1, H=2)
    host = inputs.dense_cache(w, n_threads=16)
    job = Job(w, host)
    zeros = np.zeros((w.units, w.T), np.float32)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, zeros, [0, 1])


def test_config3_full_size(oracle):
    """Config 3 at full size (28 layers x 4 KV heads = 112 units of 131072 positions), the launch shapes
    `bench.py --config 3` times: properties over every unit, element-by-element parity on two of them."""
    w = inputs.CONFIGS[3]
    host = inputs.dense_cache(w, n_threads=16)
    job = Job(w, host)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), [5, w.units - 1])


@pytest.fixture(scope="module")
def cfg4_host():
    w = inputs.CONFIGS[4]
    host = inputs.dense_cache(w, n_threads=16)
    host["K_dev"], host["V_dev"] = to_dev(host["K"]), to_dev(host["V"])      # one upload for the 60 jobs below
    return w, host


@pytest.mark.parametrize("scorer", ["last", "mean", "keydiff", "expected", "expected_vnorm"])
def test_config4_scorer_sweep(oracle, scorer, cfg4_host):
    """Config 4 at its stated shapes (256 units x 32768 positions, the launch shapes `bench.py --scorer ...`
    times): scorer x S in {1,4,16,64} x budget in T/{8,16,32}.  Per combination: properties over all units
    and the whole event against the oracle on 16 sampled units; the scores of each scorer against the oracle
    once, on 32 units; S = 1 against a stable global top-k on every unit."""
    sc = {"last": B.SCORER_LAST_QUERY, "mean": B.SCORER_MEAN_WINDOW, "keydiff": B.SCORER_KEYDIFF,
          "expected": B.SCORER_EXPECTED, "expected_vnorm": B.SCORER_EXPECTED_VNORM}[scorer]
    base, host = cfg4_host
    assert base.units == 256 and base.T == 32768
    zeros = np.zeros((base.units, base.T), np.float32)
    rng = np.random.default_rng(4)
    first = True
    for S in (1, 4, 16, 64):
        for ratio in (8, 16, 32):
            w = base.scaled(S=S, budget=base.T // ratio)
            job = Job(w, host, scorer=sc)
            job.step()
            torch.cuda.synchronize()
            check_properties_all_units(job)
            sample = sorted(rng.choice(w.units, size=32 if first else 16, replace=False).tolist())
            check_units(oracle, job, host, zeros, sample, scorer=sc, check_scores=first)
            first = False
            if S == 1:
                g = to_host(job.intermediates().g)[:, :w.T]
                idx = to_host(job.idx)
                for i in range(w.units):
                    order = np.argsort(-g[i].astype(np.float64), kind="stable")
                    np.testing.assert_array_equal(idx[i], np.sort(order[: w.budget]))
            del job
            torch.cuda.empty_cache()


@pytest.mark.parametrize("options", [{}, dict(n_sink=4, n_last=16, causal=True), dict(paged=True)])
def test_redundancy_scorer_step(oracle, options):
    """The whole event with the redundancy-aware plug-in scorer (the R-KV-style score): segments and quotas from
    the usage as always, the in-segment ranking from the redundancy-aware score; every unit against the oracle."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=3000, budget=256, S=8, n_spans=5, span_len=(16, 200), **options)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host, scorer=B.SCORER_REDUNDANCY)
    job.step()
    torch.cuda.synchronize()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)), scorer=B.SCORER_REDUNDANCY)
    # the ranking differs from plain attention: the two scorers keep different sets
    job2 = Job(w, host, scorer=B.SCORER_MEAN_WINDOW)
    job2.step()
    torch.cuda.synchronize()
    assert not torch.equal(job.idx, job2.idx)


def test_budget_at_least_length_keeps_everything(oracle):
    w = inputs.CONFIGS[0].scaled(T=700, budget=1024, H=2)
    host = inputs.dense_cache(w, n_threads=2)
    job = Job(w, host)
    job.step()
    torch.cuda.synchronize()
    idx = to_host(job.idx)
    for i in range(w.units):
        np.testing.assert_array_equal(idx[i, :700], np.arange(700))
        assert (idx[i, 700:] == -1).all()
    assert (to_host(job.n_kept) == 700).all()
    np.testing.assert_array_equal(to_host(job.Kd).reshape(w.units, 700, w.D), host["K"].reshape(w.units, 700, w.D))
    check_units(oracle, job, host, np.zeros((w.units, 700), np.float32), [0, 1])


def test_ema_zero_reproduces_raw_boundaries(oracle):
    w = inputs.CONFIGS[0].scaled(T=3000, H=2, lam=0.0)
    host = inputs.dense_cache(w, n_threads=2)
    credit = np.random.default_rng(0).random((w.units, w.T)).astype(np.float32)
    job = Job(w, host, credit=credit)
    job.step()
    torch.cuda.synchronize()
    inter = job.intermediates()
    u = to_host(inter.u)[:, :w.T]
    for i in range(w.units):
        m = oracle.mass(u[i], w.eps)
        assert_close_rel(to_host(inter.m_used)[i, :w.T], m, what="m_used == m_cur")
        np.testing.assert_array_equal(to_host(inter.bounds)[i], oracle.segment(to_host(inter.m_used)[i, :w.T], w.S)[0])


@pytest.mark.parametrize("n_sink,n_last", [(4, 32), (0, 128), (4, 0), (4, 3000), (600, 0)])
def test_must_keep_step(oracle, n_sink, n_last):
    """Sinks and a recent suffix always kept, budget shared by the segments reduced first, duplicates
    backfilled (Sec. 3.3 must-keep rules): whole step against the oracle, bf16, several units."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=6000, budget=512, S=8, n_spans=6, span_len=(32, 300),
                                 n_sink=n_sink, n_last=n_last)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)))


@pytest.mark.parametrize("scorer", ["mean", "last"])
def test_causal_must_keep_step(oracle, scorer):
    """The decoder-facing configuration: causal window, sinks and recent suffix, whole step."""
    sc = {"mean": B.SCORER_MEAN_WINDOW, "last": B.SCORER_LAST_QUERY}[scorer]
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=6000, budget=512, S=8, n_spans=6, span_len=(32, 300),
                                 n_sink=4, n_last=32, causal=True)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host, scorer=sc)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)), scorer=sc)


@pytest.mark.parametrize("delta,l_min,l_max,pool", [(0.1, 16, 256, 5), (0.05, 0, 128, 0), (0.1, 64, 0, 3),
                                                     (0.02, 16, 256, 7)])
def test_segmentation_as_printed_step(oracle, delta, l_min, l_max, pool):
    """Target segment mass with split / merge and pooled usage (Sec. 3.3; App. A), together with the
    must-keep set and the causal window: the configuration the paper's hyper-parameter table describes."""
    T = 6000
    cap = int(np.ceil(1 / delta)) + 1 + (T // l_max if l_max else 0)
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=T, budget=512, S=cap, n_spans=6, span_len=(32, 300),
                                 n_sink=4, n_last=32, causal=True, seg_delta=delta, l_min=l_min, l_max=l_max,
                                 pool_kernel=pool)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)))
    # a second event on the same cache: the credit is now non-zero
    credit_before = to_host(job.credit).copy()
    job.step()
    check_units(oracle, job, host, credit_before[:, :w.T], [0, w.units - 1])


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("options", [{}, {"n_sink": 4, "n_last": 32, "causal": True}])
def test_empty_and_tiny_sequences_in_a_batch(oracle, paged, options):
    """A batch whose sequences hold 0, 1, 5, 31, 300 and 2049 positions (budget 256, window 32): the
    empty one keeps nothing and writes nothing, the short ones keep everything, the rest match the oracle."""
    lens = np.array([0, 1, 5, 31, 300, 2049], np.int32)
    w = inputs.CONFIGS[2].scaled(L=1, H=2, B=len(lens), T=2049, T_min=2049, budget=256, S=8, n_spans=4,
                                 span_len=(16, 200), paged=paged, **options)
    host = inputs.dense_cache(w, n_threads=4)
    host["seq_lens"][:] = lens
    job = Job(w, host)
    sentinel = 123.0
    job.credit.fill_(0.0)
    job.credit_dst.fill_(sentinel)
    job.step()
    torch.cuda.synchronize()
    nk, idx, cdst = to_host(job.n_kept), to_host(job.idx), to_host(job.credit_dst)
    for i, (l, b, h) in enumerate(unit_list(w)):
        T = int(lens[b])
        assert nk[i] == min(T, w.budget)
        assert (idx[i, nk[i]:] == -1).all()
        if T <= w.budget:
            np.testing.assert_array_equal(idx[i, :T], np.arange(T))
        assert (cdst[i, nk[i]:] == sentinel).all()               # nothing written beyond the kept count
    full = [i for i, (l, b, h) in enumerate(unit_list(w)) if lens[b] > 0]
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), full)


@pytest.mark.parametrize("delta,l_min,l_max,pool", [(0.1, 16, 256, 5), (0.02, 0, 0, 3)])
def test_segmentation_as_printed_long_cache_step(oracle, delta, l_min, l_max, pool):
    """The same on a cache of 40000 positions: more groups of positions than the one-workgroup-per-unit
    kernel keeps run-end prefixes for, so the masses of the moved segments are summed from m_used."""
    T = 40000
    cap = int(np.ceil(1 / delta)) + 1 + (T // l_max if l_max else 0)
    w = inputs.CONFIGS[1].scaled(L=1, H=2, T=T, budget=1024, S=cap, n_spans=12, span_len=(64, 600),
                                 n_sink=4, n_last=32, causal=True, seg_delta=delta, l_min=l_min, l_max=l_max,
                                 pool_kernel=pool)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)))


@pytest.mark.parametrize("S,pool,n_sink,n_last", [(8, 3, 0, 0), (16, 5, 4, 32), (100, 0, 0, 0), (200, 0, 4, 16)])
def test_fixed_thresholds_with_pooling_or_many_segments_step(oracle, S, pool, n_sink, n_last):
    """Thresholds k/S with pooled usage, or with more than 64 segments: the general form of the
    one-workgroup-per-unit mass kernel without the split / merge pass, and the many-segment quota."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=9000, budget=1024, S=S, n_spans=6, span_len=(32, 300),
                                 n_sink=n_sink, n_last=n_last, pool_kernel=pool)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)))
    credit_before = to_host(job.credit).copy()
    job.step()
    check_units(oracle, job, host, credit_before[:, :w.T], [0, w.units - 1])


@pytest.mark.parametrize("dtype,paged", [("bf16", False), ("f32", False), ("bf16", True)])
def test_head_dim_64_step(oracle, dtype, paged):
    """Whole step on caches with 64 channels per head (rows of 128 / 256 bytes), dense and paged."""
    if paged:
        w = inputs.CONFIGS[2].scaled(L=1, B=6, H=3, D=64, T=3000, T_min=700, n_spans=4, span_len=(16, 100), budget=256,
                                     n_sink=4, n_last=16)
    else:
        w = inputs.CONFIGS[1].scaled(L=2, H=3, D=64, dtype=dtype, T=5000, budget=512, S=8, n_spans=6, span_len=(32, 300))
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, job.t_max), np.float32), list(range(min(w.units, 8))))


def test_causal_paged_ragged(oracle):
    w = inputs.CONFIGS[2].scaled(L=1, B=8, H=4, causal=True)
    host = inputs.dense_cache(w, n_threads=8)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, job.t_max), np.float32), [0, 1, w.units // 2, w.units - 1])


def test_must_keep_paged_ragged(oracle):
    w = inputs.CONFIGS[2].scaled(L=1, B=8, H=4, n_sink=4, n_last=64)
    host = inputs.dense_cache(w, n_threads=8)
    job = Job(w, host)
    job.step()
    check_properties_all_units(job)
    check_units(oracle, job, host, np.zeros((w.units, job.t_max), np.float32), [0, 1, w.units // 2, w.units - 1])


@pytest.mark.parametrize("scorer", [B.SCORER_MEAN_WINDOW, B.SCORER_LAST_QUERY, B.SCORER_KEYDIFF])
def test_both_score_paths(oracle, scorer):
    """ams_params.score_path pins how the softmax statistics are formed: K held on chip and read once, or
    streamed twice.  Both compute the same event (ragged tail, several workgroups per unit, more units than
    clusters run at once would need), and the kernel labels show that the pinned path really ran."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=5000, budget=512, S=8, n_spans=6, span_len=(32, 300))
    host = inputs.dense_cache(w, n_threads=4)
    us = {}
    for path, ran, not_ran in ((B.SCORE_PATH_ONE_READ, "score_oneread", "score_stats"),
                               (B.SCORE_PATH_TWO_SWEEPS, "score_stats", "score_oneread")):
        job = Job(w, host, scorer=scorer, score_path=path)
        B.ams_profile_begin()
        job.step()
        labels = [k for k, _ in B.ams_profile_end()]
        assert ran in labels and not_ran not in labels
        check_properties_all_units(job)
        check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)), scorer=scorer)
        us[path] = job.intermediates().u[:, :w.T].cpu().numpy()
    np.testing.assert_allclose(us[B.SCORE_PATH_ONE_READ], us[B.SCORE_PATH_TWO_SWEEPS], rtol=2e-5, atol=1e-12)


def test_one_read_path_reports_an_expired_wait():
    """The one path whose workgroups wait for one another: with the bound of its waits set to a single poll
    (from the host; every kernel still runs to its end) a member that is not the last to arrive gives up, the
    step says so with n_kept = -1 for every unit, and the next step with the built-in bound is whole again."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=5000, budget=512, S=8, n_spans=6, span_len=(32, 300))
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host, score_path=B.SCORE_PATH_ONE_READ)
    B.ams_debug_set_wait_limit(1)
    try:
        job.step()
        torch.cuda.synchronize()
        assert (job.n_kept.cpu().numpy() == -1).all()
    finally:
        B.ams_debug_set_wait_limit(0)
    with pytest.raises(B.AmsError):
        B.ams_debug_set_wait_limit(-1)
    job.credit.zero_()
    job.step()
    torch.cuda.synchronize()
    assert (job.n_kept.cpu().numpy() == w.budget).all()
    check_properties_all_units(job)


@pytest.mark.parametrize("scorer", [B.SCORER_MEAN_WINDOW, B.SCORER_LAST_QUERY, B.SCORER_KEYDIFF])
@pytest.mark.parametrize("dtype,D,G,W,T,paged", [("bf16", 128, 4, 32, 2176, False), ("bf16", 128, 4, 32, 4096, False),
                                                  ("f32", 128, 1, 8, 1280, False), ("bf16", 64, 2, 16, 3000, False),
                                                  ("f32", 64, 3, 5, 257, False), ("bf16", 128, 4, 32, 1, False),
                                                  ("bf16", 128, 4, 32, 2500, True)])
def test_one_launch_score_path(oracle, scorer, dtype, D, G, W, T, paged):
    """Short caches through the pinned one-launch scorer (one workgroup walks a unit's keys twice): the whole
    event against the oracle on every unit, and the usage equal to the two sweeps' to rounding."""
    w = inputs.CONFIGS[1].scaled(L=2, H=3, T=T, D=D, G=G, W=W, dtype=dtype, budget=min(256, T), S=8, n_spans=3,
                                 span_len=(8, 100), paged=paged)
    host = inputs.dense_cache(w, n_threads=4)
    us = {}
    for path, ran in ((B.SCORE_PATH_ONE_LAUNCH, "score_unit"), (B.SCORE_PATH_TWO_SWEEPS, "score_stats")):
        job = Job(w, host, scorer=scorer, score_path=path)
        B.ams_profile_begin()
        job.step()
        labels = [k for k, _ in B.ams_profile_end()]
        assert ran in labels and ("score_stats" in labels) == (ran == "score_stats")
        check_properties_all_units(job)
        check_units(oracle, job, host, np.zeros((w.units, w.T), np.float32), list(range(w.units)), scorer=scorer)
        us[path] = job.intermediates().u[:, :w.T].cpu().numpy()
    np.testing.assert_allclose(us[B.SCORE_PATH_ONE_LAUNCH], us[B.SCORE_PATH_TWO_SWEEPS], rtol=2e-5, atol=1e-12)


def test_one_launch_path_ragged_batch_and_auto(oracle):
    """A ragged batch (lengths 0, 1, 31, 300, 2049, 4096) through the one-launch scorer; with at least 128 units
    the library takes that path by itself, with fewer it keeps the two sweeps."""
    w = inputs.CONFIGS[2].scaled(L=1, B=6, H=2, T=4096, T_min=None, paged=False, budget=128, S=4, n_spans=2,
                                 span_len=(4, 40))
    host = inputs.dense_cache(w, n_threads=4)
    host["seq_lens"] = np.array([0, 1, 31, 300, 2049, 4096], np.int32)
    job = Job(w, host, score_path=B.SCORE_PATH_ONE_LAUNCH)
    job.step()
    torch.cuda.synchronize()
    nk, idx = to_host(job.n_kept), to_host(job.idx)
    assert (nk[:2] == 0).all() and (idx[:2] == -1).all()               # the empty sequence keeps nothing
    check_units(oracle, job, host, np.zeros((w.units, job.t_max), np.float32), [i for i in range(w.units) if i >= 2])
    for L, label in ((16, "score_unit"), (4, "score_stats")):          # 128 units / 32 units
        wa = inputs.CONFIGS[1].scaled(L=L, H=8, T=1500, budget=128, S=4, n_spans=2, span_len=(4, 40))
        ja = Job(wa, inputs.dense_cache(wa, n_threads=8))
        B.ams_profile_begin()
        ja.step()
        assert label in [k for k, _ in B.ams_profile_end()]
        check_properties_all_units(ja)


def test_one_read_path_says_when_it_does_not_apply():
    """A pinned one-read path is refused (AMS_ERR_UNSUPPORTED, nothing half done) where only the two sweeps
    exist: fp32 caches, the causal window, the moment-based scorers."""
    base = inputs.CONFIGS[1].scaled(L=1, H=2, T=1000, budget=128, S=4, n_spans=2, span_len=(16, 64))
    for w, scorer in ((base.scaled(dtype="f32"), B.SCORER_MEAN_WINDOW), (base.scaled(causal=True), B.SCORER_MEAN_WINDOW),
                      (base, B.SCORER_EXPECTED)):
        host = inputs.dense_cache(w, n_threads=2)
        job = Job(w, host, scorer=scorer, score_path=B.SCORE_PATH_ONE_READ)
        with pytest.raises(B.AmsError) as err:
            job.step()
        assert err.value.status == B.ERR_UNSUPPORTED
        Job(w, host, scorer=scorer, score_path=B.SCORE_PATH_AUTO).step()      # the library's own choice works
    for w, scorer in ((base.scaled(T=5000), B.SCORER_MEAN_WINDOW), (base.scaled(causal=True), B.SCORER_MEAN_WINDOW),
                      (base, B.SCORER_EXPECTED)):                             # the one-launch path: short caches only
        job = Job(w, inputs.dense_cache(w, n_threads=2), scorer=scorer, score_path=B.SCORE_PATH_ONE_LAUNCH)
        with pytest.raises(B.AmsError) as err:
            job.step()
        assert err.value.status == B.ERR_UNSUPPORTED
    torch.cuda.synchronize()


def test_step_under_graph_capture(oracle):
    """The fused call allocates nothing and never waits for the stream, so it can be recorded into a
    HIP graph; every replay (with eager work between replays) gives the eager result bit for bit."""
    w = inputs.CONFIGS[1].scaled(L=2, H=4, T=5000, budget=512, S=8, n_spans=6, span_len=(32, 300), n_sink=4,
                                 n_last=32, causal=True)
    host = inputs.dense_cache(w, n_threads=4)
    job = Job(w, host)
    job.step()                                             # eager: also sets the kernels' attributes once
    torch.cuda.synchronize()
    want = (job.idx.clone(), job.Kd.clone(), job.credit.clone(), job.credit_dst.clone())
    credit0 = torch.zeros_like(job.credit)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    job.credit.copy_(credit0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        job.step(torch.cuda.current_stream())
    for _ in range(3):
        job.credit.copy_(credit0)                          # eager work between the replays
        job.idx.fill_(-7)
        job.Kd.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(job.idx, want[0]) and torch.equal(job.Kd, want[1])
        assert torch.equal(job.credit, want[2]) and torch.equal(job.credit_dst, want[3])
