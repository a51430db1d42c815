#!/usr/bin/env python3
"""Throughput of the fused AMS compression step on one MI355X.

A step is one whole compression event (score -> mass -> EMA -> prefix sum / boundaries -> quotas ->
segmented top-k -> gather-compact) over every (layer, KV head) of a synthetic cache with the shapes of
the 32k-context configuration: 32 layers x 8 KV heads, group 4, head_dim 128, bf16, T = 32768, query
window 32, budget 2048, S = 16, lambda = 0.9.  Inputs are resident in HBM before the timed region.
Every timed step runs at T = 32768 against the same source cache (the destination is a separate
buffer); the credit vector persists across steps at full length and a different query window is
used from step to step, so each step does the full work of an event.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E, published


def _token_sums(w, lens):
    """(sum of the sequence lengths, sum of the kept counts) over the batch."""
    if lens is None:
        return w.B * w.T, w.B * min(w.budget, w.T)
    return int(sum(int(t) for t in lens)), int(sum(min(w.budget, int(t)) for t in lens))


def algorithmic_bytes(w, lens=None):
    """Bytes one event must move over all units: K read once for scoring, kept K/V rows read and written,
    three fp32 vector passes (u write + read, credit read), index and credit' writes."""
    e = w.elem_bytes
    tok, kept = _token_sums(w, lens)
    return (tok * w.D * e + 4 * kept * w.D * e + 4 * tok * 3 + 4 * kept * 2) * w.L * w.H


def kernel_bytes(label, w, lens=None):
    """Algorithmic bytes of one launch of a kernel over all units (what it must read + write)."""
    e, D = w.elem_bytes, w.D
    tok, kept = _token_sums(w, lens)
    per_layer_head = {
        "score_stats": tok * D * e,                       # K stream
        "score_usage": tok * D * e + 4 * tok,             # K stream + u
        "score_reduce": 0,
        "score_oneread": tok * D * e + 4 * tok * 2,       # K stream once, u out, old credit in (for its sum)
        "score_unit": tok * D * e + 4 * tok * 2,          # short caches: K counted once (the second walk hits the caches)
        "khat_sum": tok * D * e,                          # K stream (sum of the normalised keys)
        "mean_cos": tok * D * e + 4 * tok,                # K stream + the mean cosine per key
        "esoftmax_part": 4 * tok,                         # the mean cosines once more (softmax statistics)
        "redundancy_combine": 4 * tok * 3,                # u, mean cosine in; g out
        "keysum": tok * D * e,                            # K stream (mean key)
        "keydiff": tok * D * e + 4 * tok,                 # K stream + g
        "mass_ema": 4 * tok * 4,                          # u, credit in; credit, m_used out
        "unit_mass": 4 * tok * 4,                         # the same, with the scan and the quotas in the same launch
        "segment_scan": 4 * tok,                          # m_used in
        "quota": 0,
        "select": 4 * tok + 4 * kept,                     # g in, idx out
        "compact": 4 * kept * D * e + 4 * kept * 3,       # K,V rows in + out, idx, credit gather
    }.get(label, 0)
    return per_layer_head * w.L * w.H


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="workload number (1 = the headline 32k configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=256, help="units of the workload the CPU oracle is timed on")
    ap.add_argument("--n-sink", type=int, default=0, help="must-keep sinks (not part of the headline workload)")
    ap.add_argument("--n-last", type=int, default=0, help="must-keep recent suffix (not part of the headline workload)")
    ap.add_argument("--causal", action="store_true", help="causal query window (not part of the headline workload)")
    ap.add_argument("--seg-delta", type=float, default=0.0, help="target segment mass as printed, with --l-min/--l-max "
                    "(not part of the headline workload; the segment arrays get the capacity they need)")
    ap.add_argument("--l-min", type=int, default=0)
    ap.add_argument("--l-max", type=int, default=0)
    ap.add_argument("--pool", type=int, default=0, help="average-pooling kernel of the usage (odd)")
    ap.add_argument("--scorer", default="mean_window",
                    choices=["mean_window", "last_query", "keydiff", "expected", "expected_vnorm", "redundancy"],
                    help="base scorer (the headline workload uses mean_window)")
    ap.add_argument("--score-path", default="auto", choices=["auto", "two_sweeps", "one_read", "one_launch"],
                    help="ams_params.score_path: how the softmax statistics are formed (the headline line uses auto)")
    ap.add_argument("--seq-len", type=int, default=0,
                    help="run the dense workload at this cache length instead of its own (e.g. budget + appended tokens: "
                         "the short event of the literal trajectory as the main workload of a profiling run)")
    ap.add_argument("--no-small-event", action="store_true",
                    help="skip the short event of the literal trajectory (profiling runs: one workload per kernel name)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that a counter run of this "
                         "command can be scaled: see profiles/")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (units are independent; there is no multi-GPU path). "
                 "Run with --gpus 1.")

    import numpy as np
    import torch
    from paper_2605_23200_amd import binding as B
    from paper_2605_23200_amd import inputs
    from paper_2605_23200_amd.harness import Job

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()                                   # fails loudly if the HIP library is not built
    w = inputs.CONFIGS[args.config].scaled(n_sink=args.n_sink, n_last=args.n_last, causal=args.causal,
                                           pool_kernel=args.pool)
    if args.seq_len > 0:
        if w.paged or not (w.W <= args.seq_len <= w.T):
            sys.exit("bench.py: --seq-len is for the dense workloads, between the window and the configured length")
        w = w.scaled(T=args.seq_len, n_spans=max(1, w.n_spans * args.seq_len // w.T))
    if args.scorer == "redundancy":
        args.no_cpu_baseline = True       # its definition is quadratic in the cache length: hours on the host at 32k
    if args.seg_delta > 0:
        import math
        cap = math.ceil(1 / args.seg_delta) + 1 + (w.T // args.l_max if args.l_max else 0)
        w = w.scaled(seg_delta=args.seg_delta, l_min=args.l_min, l_max=args.l_max, S=cap)
    t0 = time.time()
    scorer_id = {"mean_window": B.SCORER_MEAN_WINDOW, "last_query": B.SCORER_LAST_QUERY,
                 "keydiff": B.SCORER_KEYDIFF, "expected": B.SCORER_EXPECTED,
                 "expected_vnorm": B.SCORER_EXPECTED_VNORM, "redundancy": B.SCORER_REDUNDANCY}[args.scorer]
    score_path = {"auto": B.SCORE_PATH_AUTO, "two_sweeps": B.SCORE_PATH_TWO_SWEEPS,
                  "one_read": B.SCORE_PATH_ONE_READ, "one_launch": B.SCORE_PATH_ONE_LAUNCH}[args.score_path]
    n_q = 4
    lens = None
    if w.paged:
        # the paged, ragged configuration is far too large to draw on the host: lengths and block tables are
        # the seeded ones, the values are drawn on the device (no oracle leg, no planted spans)
        from paper_2605_23200_amd.harness import DeviceFilledPagedJob
        host = None
        job = DeviceFilledPagedJob(w, scorer=scorer_id)
        lens = job.lens_h
        q_windows = [job.Q] + [torch.randn_like(job.Q, dtype=torch.float32).to(job.Q.dtype) for _ in range(n_q - 1)]
        args.no_cpu_baseline = True
    else:
        if w.T_min is not None:
            sys.exit("bench.py: ragged workloads are benchmarked in the paged layout only")
        host = inputs.dense_cache(w, n_threads=16)
        job = Job(w, host, scorer=scorer_id, score_path=score_path)
        q_windows = [job.Q] + [torch.empty_like(job.Q) for _ in range(n_q - 1)]
        for e in range(1, n_q):
            Q = np.zeros_like(host["Q"])
            for (l, b, h) in inputs.unit_ids(w):
                Q[l, b, h * w.G:(h + 1) * w.G] = inputs.unit_q(w, l, b, h, e)
            q_windows[e].copy_(torch.from_numpy(Q.view(np.int16) if Q.dtype == np.uint16 else Q))
    setup_s = time.time() - t0
    stream = torch.cuda.current_stream()

    def one_step(i):
        job.Q = q_windows[i % n_q]
        job.step(stream)

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-kernel durations: HIP events recorded by the library before every launch, same stream
    B.ams_profile_begin()
    for i in range(args.steps):
        one_step(i)
    marks = B.ams_profile_end(stream)
    per = {}
    for label, ms in marks:
        per.setdefault(label, []).append(ms)
    kern = {k: sum(v) / len(v) for k, v in per.items()}
    # one figure per step of that region: the sum of its kernels' intervals
    n_prof = min(len(v) for v in per.values())
    step_sums = sorted(sum(per[k][i] for k in per) for i in range(n_prof))
    dom = max(kern, key=kern.get)
    dom_bytes = kernel_bytes(dom, w, lens)
    achieved = dom_bytes / (kern[dom] * 1e-3) / 1e9

    # the ceiling a plain device copy reaches in the same run (1 GiB read + 1 GiB written)
    src_c = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
    dst_c = torch.empty_like(src_c)
    dst_c.copy_(src_c)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst_c.copy_(src_c)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * src_c.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src_c, dst_c

    # the literal trajectory's later events are short (kept rows + appended tokens): launch-bound
    small_ms = None
    if w.n_append > 0 and not w.paged and not args.no_small_event:
        ws_small = w.scaled(T=w.budget + w.n_append, n_spans=max(1, w.n_spans * (w.budget + w.n_append) // w.T))
        job_s = Job(ws_small, inputs.dense_cache(ws_small, n_threads=16), scorer=scorer_id, score_path=score_path)
        for _ in range(5):
            job_s.step(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(50):
            job_s.step(stream)
        torch.cuda.synchronize()
        small_ms = (time.perf_counter() - t0) / 50 * 1e3
        B.ams_profile_begin()
        for _ in range(20):
            job_s.step(stream)
        per_s = {}
        for label, ms in B.ams_profile_end(stream):
            per_s.setdefault(label, []).append(ms)
        small_kern = {k: round(sum(v) / len(v), 4) for k, v in per_s.items()}
        del job_s

    if args.calibrate_copy:
        src_c = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst_c = torch.empty_like(src_c)
        for _ in range(3):
            dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c

    step_bytes = algorithmic_bytes(w, lens)
    eff_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_config{args.config}.json")
    if os.path.exists(tpath):          # HBM bytes per launch from rocprofv3 --pmc runs of this command
        with open(tpath) as f:
            traffic = json.load(f).get("kernels", {}).get(dom, {}).get("hbm_bytes_per_launch")

    out = {
        "metric": "ams_compress_steps_per_sec", "value": round(1e3 / ms_per_step, 3), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"config{args.config}: {w.L}L x {w.H} KV heads, group {w.G}, D {w.D}, {w.dtype}, "
                               f"T {w.T}{'' if lens is None else f' (ragged from {w.T_min}, paged, device-drawn values)'}, window {w.W}, budget {w.budget}, S {w.S}, lambda {w.lam}, "
                               f"{'no' if lens is not None else w.n_spans} planted spans, seed {w.seed}; steady-state events at full T"
                               + (f"; must-keep {w.n_sink}+{w.n_last}" if w.n_sink or w.n_last else "")
                               + ("; causal window" if w.causal else "")
                               + (f"; Delta {w.seg_delta} L {w.l_min}/{w.l_max}" if w.seg_delta else "")
                               + (f"; pool {w.pool_kernel}" if w.pool_kernel > 1 else ""),
                   "units": w.units, "scorer": args.scorer, "score_path": args.score_path},
        "effective_GBps": round(eff_gbps, 1), "algorithmic_bytes_per_step": step_bytes,
        "hbm_peak_frac": round(eff_gbps / HBM_PEAK_GBPS, 4),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel_ms": round(kern[dom], 4), "algorithmic_bytes_per_launch": dom_bytes},
        "kernel_ms": {k: round(v, 4) for k, v in kern.items()},
        "stage_GBps": {k: round(kernel_bytes(k, w, lens) / (v * 1e-3) / 1e9, 1) for k, v in kern.items()
                       if kernel_bytes(k, w, lens) > 0},
        "step_ms_median": round(step_sums[len(step_sums) // 2], 4), "step_ms_min": round(step_sums[0], 4),
        "copy_GBps": round(copy_gbps, 1),
        "small_event": None if small_ms is None else
        {"T": w.budget + w.n_append, "ms_per_step": round(small_ms, 4), "kernel_ms": small_kern,
         "note": "a later event of the literal trajectory: kept rows + appended tokens"},
        "setup_s": round(setup_s, 1),
    }

    if not args.no_cpu_baseline:
        from oracle import ams_oracle as O
        n_units = min(args.cpu_units, w.units)
        ids = inputs.unit_ids(w)[:n_units]
        Qf = np.stack([inputs.as_f32(host["Q"][l, b, h * w.G:(h + 1) * w.G]).reshape(-1, w.D) for l, b, h in ids])
        Kf = np.stack([inputs.as_f32(host["K"][l, b, h]) for l, b, h in ids])
        Kr = np.stack([host["K"][l, b, h] for l, b, h in ids])
        Vr = np.stack([host["V"][l, b, h] for l, b, h in ids])
        credit = np.zeros((n_units, w.T), np.float32)
        n_threads = min(16, os.cpu_count() or 1)
        t0 = time.perf_counter()
        _, _, used = O.compress_many(np.ascontiguousarray(Qf), np.ascontiguousarray(Kf), credit, G=w.G, W=w.W,
                                     budget=w.budget, S=w.S, lam=w.lam, beta=w.beta, eps=w.eps, q_min=w.q_min,
                                     n_threads=n_threads, K_rows=Kr, V_rows=Vr, scorer=scorer_id,
                                     V=np.ascontiguousarray(np.stack([inputs.as_f32(host["V"][l, b, h]) for l, b, h in ids]))
                                     if scorer_id == B.SCORER_EXPECTED_VNORM else None, n_sink=w.n_sink, n_last=w.n_last,
                                     causal=w.causal, delta=w.seg_delta, l_min=w.l_min, l_max=w.l_max,
                                     pool_kernel=w.pool_kernel)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n_units / cpu_s / w.units, 5), "unit": "steps/s", "cores": used,
                               "kind": "oracle", "host_cpus": os.cpu_count(),
                               "sample": f"first {n_units} of {w.units} units of the same workload, one event, "
                                         f"{cpu_s:.1f} s wall, scaled linearly to a whole step"}
        # one core on the small fp32 configuration, for scale
        w0 = inputs.CONFIGS[0]
        h0 = inputs.dense_cache(w0, n_threads=4)
        ids0 = inputs.unit_ids(w0)
        Q0 = np.ascontiguousarray(np.stack([inputs.as_f32(h0["Q"][l, b, h * w0.G:(h + 1) * w0.G]).reshape(-1, w0.D)
                                            for l, b, h in ids0]))
        K0 = np.ascontiguousarray(np.stack([inputs.as_f32(h0["K"][l, b, h]) for l, b, h in ids0]))
        t0 = time.perf_counter()
        O.compress_many(Q0, K0, np.zeros((w0.units, w0.T), np.float32), G=w0.G, W=w0.W, budget=w0.budget, S=w0.S,
                        lam=w0.lam, beta=w0.beta, eps=w0.eps, q_min=w0.q_min, n_threads=1)
        out["cpu_baseline"]["config0_one_core_steps_per_s"] = round(1.0 / (time.perf_counter() - t0), 3)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
