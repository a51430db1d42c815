"""Retention diagnostics on synthetic trajectories (App. "Additional Mechanistic Diagnostics").

The paper reports, for its own models and datasets, a region wipe-out rate, the retained-set IoU
between consecutive compression events and the number / length of adaptive segments.  None of that
data exists here; this module re-creates the *metrics* on the seeded synthetic caches of
`inputs.py` so that segment-wise allocation (S > 1) can be compared with a global top-k (S = 1) and
the EMA credit switched on and off.  The paper does not define the wipe-out rate precisely.  Two
readings are computed here: over the PLANTED SPANS of the synthetic cache (the stand-ins for the
paper's dense-attention regions) -- a span is wiped out by an event when it had tokens in the cache
before the event and none after it, and the cumulative figure is the fraction of planted spans with
no token left after the last event -- and over fixed windows of `region` consecutive original
positions, the same way.

The metric functions are plain numpy on index sets.  `run_trajectory` drives the HIP library through
the same C ABI as everything else (there is no other implementation of the method in this package).
"""
import argparse
import json
from dataclasses import dataclass, field
from typing import List

import numpy as np


def region_wipeout_rate(present: np.ndarray, kept: np.ndarray, region: int) -> float:
    """present, kept: original positions in the cache before / after an event (kept is a subset).
    Fraction of the regions touched by `present` that `kept` does not touch."""
    before = np.unique(np.asarray(present) // region)
    after = np.unique(np.asarray(kept) // region)
    if len(before) == 0:
        return 0.0
    return float(len(np.setdiff1d(before, after, assume_unique=True)) / len(before))


def span_wipeout(spans: np.ndarray, present: np.ndarray, kept: np.ndarray):
    """spans: rows (start, stop, ...) in original positions.  Returns (spans that had a token in `present`,
    spans among those with no token in `kept`)."""
    present, kept = np.sort(np.asarray(present)), np.sort(np.asarray(kept))
    had = gone = 0
    for row in np.asarray(spans):
        st, en = int(row[0]), int(row[1])
        n_before = np.searchsorted(present, en) - np.searchsorted(present, st)
        if n_before > 0:
            had += 1
            gone += int(np.searchsorted(kept, en) - np.searchsorted(kept, st) == 0)
    return had, gone


def retained_iou(kept_a: np.ndarray, kept_b: np.ndarray) -> float:
    """Intersection over union of two retained sets of original positions."""
    a, b = np.unique(kept_a), np.unique(kept_b)
    union = len(np.union1d(a, b))
    return float(len(np.intersect1d(a, b, assume_unique=True)) / union) if union else 1.0


def retention_profile(present: np.ndarray, kept: np.ndarray, bins: int = 10) -> np.ndarray:
    """Fraction of the tokens kept in each of `bins` equal slices of the cache (by rank in `present`)."""
    present = np.sort(np.asarray(present))
    is_kept = np.isin(present, kept)
    edges = np.linspace(0, len(present), bins + 1).astype(int)
    return np.array([is_kept[edges[i]:edges[i + 1]].mean() if edges[i + 1] > edges[i] else 0.0 for i in range(bins)])


def segment_stats(bounds: np.ndarray):
    """bounds [S+1] of one unit -> (number of non-empty segments, their mean length)."""
    lens = np.diff(np.asarray(bounds))
    lens = lens[lens > 0]
    return int(len(lens)), float(lens.mean()) if len(lens) else 0.0


@dataclass
class EventRecord:
    present: List[np.ndarray] = field(default_factory=list)   # per unit: original positions before the event
    kept: List[np.ndarray] = field(default_factory=list)      # per unit: original positions after it
    bounds: List[np.ndarray] = field(default_factory=list)


def run_trajectory(w, *, n_events: int, scorer=None, device: str = "cuda:0") -> List[EventRecord]:
    """Compress, append `w.n_append` fresh tokens, compress again ... on the GPU, tracking the original
    position of every cached token.  The credit of kept tokens is carried, fresh tokens start at 0."""
    import torch
    from . import binding as B
    from . import inputs

    scorer = B.SCORER_MEAN_WINDOW if scorer is None else scorer
    host = inputs.dense_cache(w, n_threads=8)
    ids = inputs.unit_ids(w)

    def dev(a):
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(device)

    K, V = dev(host["K"]), dev(host["V"])
    units = w.units
    credit = torch.zeros((units, w.T), device=device)
    pos = torch.arange(w.T, device=device, dtype=torch.int64).repeat(units, 1)
    next_id = w.T
    out = []
    for e in range(n_events):
        T = K.shape[3]
        keep = min(w.budget, T)
        p = B.make_params(n_layers=w.L, batch=w.B, n_kv_heads=w.H, group=w.G, window=w.W, head_dim=w.D,
                          kv_dtype=B.F32 if w.dtype == "f32" else B.BF16, t_max=T, t_stride=T, budget=w.budget,
                          n_segments=w.S, q_min=w.q_min, ema_lambda=w.lam, ema_beta=w.beta, mass_eps=w.eps,
                          scorer=scorer, n_sink=w.n_sink, n_last=w.n_last, causal=w.causal,
                          seg_delta=w.seg_delta, l_min=w.l_min, l_max=w.l_max, pool_kernel=w.pool_kernel)
        Q = np.zeros_like(host["Q"])
        for (l, b, h) in ids:
            Q[l, b, h * w.G:(h + 1) * w.G] = inputs.unit_q(w, l, b, h, e)
        Qd = dev(Q)
        lens = torch.full((w.B,), T, dtype=torch.int32, device=device)
        Kd = torch.zeros((w.L, w.B, w.H, keep, w.D), dtype=K.dtype, device=device)
        Vd = torch.zeros_like(Kd)
        credit_dst = torch.zeros((units, w.budget), device=device)
        idx = torch.full((units, w.budget), -1, dtype=torch.int32, device=device)
        n_kept = torch.zeros(units, dtype=torch.int32, device=device)
        ws = torch.zeros(B.ams_workspace_bytes(p), dtype=torch.uint8, device=device)
        B.ams_compress_step(p, B.dense_view(K, V), lens, Qd, credit, B.dense_view(Kd, Vd), credit_dst, idx, n_kept, ws)
        torch.cuda.synchronize()
        kept_pos = torch.gather(pos, 1, idx[:, :keep].long())
        bounds = B.workspace_tensors(p, ws).bounds.cpu().numpy()
        rec = EventRecord()
        pos_h, kept_h = pos.cpu().numpy(), kept_pos.cpu().numpy()
        for i in range(units):
            rec.present.append(pos_h[i].copy())
            rec.kept.append(kept_h[i].copy())
            rec.bounds.append(bounds[i].copy())
        out.append(rec)
        if e + 1 == n_events:
            break
        # next cache: kept rows + fresh rows
        fk = np.zeros((w.L, w.B, w.H, w.n_append, w.D), host["K"].dtype)
        fv = np.zeros_like(fk)
        for (l, b, h) in ids:
            fk[l, b, h], fv[l, b, h] = inputs.unit_fresh_rows(w, l, b, h, e + 1, w.n_append)
        K = torch.cat([Kd, dev(fk)], dim=3).contiguous()
        V = torch.cat([Vd, dev(fv)], dim=3).contiguous()
        credit = torch.cat([credit_dst[:, :keep], torch.zeros((units, w.n_append), device=device)], dim=1).contiguous()
        fresh = torch.arange(next_id, next_id + w.n_append, device=device, dtype=torch.int64).repeat(units, 1)
        pos = torch.cat([kept_pos, fresh], dim=1).contiguous()
        next_id += w.n_append
    return out


def summarize(records: List[EventRecord], region: int = 64, unit_spans=None) -> dict:
    """Means over units and events of the metrics above.  unit_spans: per unit the planted spans (rows
    start, stop, ...) for the span wipe-out figures."""
    wipe, iou, nseg, slen, middle = [], [], [], [], []
    span_had = span_gone = span_total = span_dead = 0
    for e, rec in enumerate(records):
        for i in range(len(rec.kept)):
            wipe.append(region_wipeout_rate(rec.present[i], rec.kept[i], region))
            if unit_spans is not None:
                had, gone = span_wipeout(unit_spans[i], rec.present[i], rec.kept[i])
                span_had += had
                span_gone += gone
                if e + 1 == len(records):          # planted spans with nothing left at the end of the trajectory
                    span_total += len(unit_spans[i])
                    span_dead += len(unit_spans[i]) - span_wipeout(unit_spans[i], rec.kept[i], rec.kept[i])[0]
            n, m = segment_stats(rec.bounds[i])
            nseg.append(n)
            slen.append(m)
            prof = retention_profile(rec.present[i], rec.kept[i], 10)
            middle.append(prof[3:7].mean())
            if e > 0:
                iou.append(retained_iou(records[e - 1].kept[i], rec.kept[i]))
    return {"span_wipeout_rate": span_gone / span_had if span_had else None,
            "spans_lost_at_end": span_dead / span_total if span_total else None,
            "region_wipeout_rate": float(np.mean(wipe)), "retained_iou": float(np.mean(iou)) if iou else None,
            "avg_segments": float(np.mean(nseg)), "avg_segment_len": float(np.mean(slen)),
            "middle_retention": float(np.mean(middle)), "region": region}


def planted_spans(w) -> list:
    """Per unit the planted spans of its sequence (positions of the initial cache)."""
    from . import inputs
    return [inputs.spans(w, b, w.T) for (l, b, h) in inputs.unit_ids(w)]


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=0)
    ap.add_argument("--events", type=int, default=4)
    ap.add_argument("--region", type=int, default=64)
    ap.add_argument("--budget", type=int, default=0, help="override the workload's budget (0 = keep it)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = keep it)")
    args = ap.parse_args()
    from . import binding as B
    from . import inputs
    B.lib()
    base = inputs.CONFIGS[args.config]
    if base.paged or base.T_min is not None:
        raise SystemExit("dense single-length workloads only")
    if args.budget:
        base = base.scaled(budget=args.budget)
    if args.layers:
        base = base.scaled(L=args.layers)
    if base.n_append == 0:
        base = base.scaled(n_append=base.budget // 4)
    variants = {"ams": base, "global_topk (S=1)": base.scaled(S=1), "ams, no credit (lambda=0)": base.scaled(lam=0.0),
                "global_topk, no credit": base.scaled(S=1, lam=0.0)}
    for name, w in variants.items():
        for sc_name, sc in (("mean_window", B.SCORER_MEAN_WINDOW), ("last_query", B.SCORER_LAST_QUERY)):
            s = summarize(run_trajectory(w, n_events=args.events, scorer=sc), args.region, planted_spans(w))
            print(json.dumps({"variant": name, "scorer": sc_name, **s}))


if __name__ == "__main__":
    main()
