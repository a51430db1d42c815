"""Seeded synthetic KV caches shaped like long-reasoning workloads.

This module only draws inputs; it holds none of the method's arithmetic and is
the one piece of code that both the GPU tests/benchmark and the CPU oracle's
callers use.  Everything is generated on the host with numpy's counter-based
Philox generator keyed by (seed, stream), so any unit of any configuration can
be regenerated on its own, byte for byte.

Recipe: Q, K, V ~ N(0, 1).  A number of contiguous "reasoning spans" are planted
per sequence (positions shared by all layers and heads of the sequence; overlaps
allowed, the shift applied once); inside a span every key of a unit is shifted by
shift * qbar / ||qbar||, qbar being the mean of that unit's query vectors, so the
recent queries attend to the span.  Values are then rounded once to the storage
dtype (float32, or bfloat16 with round-to-nearest-even, held as uint16 bits).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Optional, Sequence, Tuple

import numpy as np

_Q_STREAM, _K_STREAM, _V_STREAM, _SPAN_STREAM, _LEN_STREAM, _TABLE_STREAM = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    B: int
    H: int            # KV heads
    G: int            # query heads per KV head
    W: int            # query window
    D: int
    dtype: str        # "f32" | "bf16"
    T: int            # KV length (max length when ragged)
    budget: int
    S: int
    lam: float
    beta: float = 0.9
    eps: float = 1e-6
    q_min: int = 1
    n_spans: int = 0
    span_len: Tuple[int, int] = (64, 256)
    span_shift: Tuple[float, float] = (1.5, 1.5)
    seed: int = 0
    T_min: Optional[int] = None   # ragged: per-sequence length uniform in [T_min, T]
    paged: bool = False
    block: int = 16
    n_events: int = 1
    n_append: int = 0
    n_sink: int = 0       # must-keep sizes (0, 0: none)
    n_last: int = 0
    causal: bool = False  # causal window with padded observations
    seg_delta: float = 0.0  # > 0: target segment mass as printed, S is then the capacity of the segment arrays
    l_min: int = 0
    l_max: int = 0
    pool_kernel: int = 0  # odd k > 1: k-point average pooling of the usage before Eq. (1)

    @property
    def N(self) -> int:
        return self.G * self.W

    @property
    def units(self) -> int:
        return self.L * self.B * self.H

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations the benchmark definition names (index = config number).
CONFIGS = {
    0: Workload("cfg0-f32-4k", L=1, B=1, H=8, G=1, W=8, D=128, dtype="f32", T=4096, budget=1024, S=8,
                lam=0.9, n_spans=6, span_len=(64, 256), seed=0, n_events=4, n_append=256),
    1: Workload("cfg1-bf16-32k", L=32, B=1, H=8, G=4, W=32, D=128, dtype="bf16", T=32768, budget=2048,
                S=16, lam=0.9, n_spans=40, span_len=(128, 1024), seed=1, n_events=8, n_append=128),
    2: Workload("cfg2-paged-ragged", L=32, B=64, H=8, G=4, W=32, D=128, dtype="bf16", T=16384,
                T_min=4096, budget=1024, S=8, lam=0.9, n_spans=40, span_len=(128, 1024), seed=2,
                paged=True, block=16),
    3: Workload("cfg3-bf16-128k", L=28, B=1, H=4, G=7, W=32, D=128, dtype="bf16", T=131072, budget=4096,
                S=32, lam=0.95, n_spans=200, span_len=(256, 2048), span_shift=(0.5, 2.0), seed=3),
    4: Workload("cfg4-scorer-sweep", L=32, B=1, H=8, G=4, W=32, D=128, dtype="bf16", T=32768, budget=2048,
                S=16, lam=0.9, n_spans=40, span_len=(128, 1024), seed=4),
}


def _rng(seed: int, *stream: int) -> np.random.Generator:
    s = 0
    for x in stream:
        s = s * 1000003 + int(x) + 1
    return np.random.Generator(np.random.Philox(key=[int(seed), s & 0xFFFFFFFFFFFFFFFF]))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return x.astype(np.float32) if dtype == "f32" else to_bf16_bits(x)


def as_f32(x: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else x


def seq_lens(w: Workload) -> np.ndarray:
    """Per-sequence KV lengths [B] (int32)."""
    if w.T_min is None:
        return np.full(w.B, w.T, np.int32)
    return _rng(w.seed, _LEN_STREAM).integers(w.T_min, w.T + 1, size=w.B).astype(np.int32)


def spans(w: Workload, b: int, T: int) -> np.ndarray:
    """Planted spans of sequence b as rows (start, stop, shift); span count scales with T / w.T."""
    r = _rng(w.seed, _SPAN_STREAM, b)
    n = max(1, round(w.n_spans * T / w.T)) if w.n_spans > 0 else 0
    out = np.zeros((n, 3), np.float64)
    for i in range(n):
        ln = int(r.integers(w.span_len[0], w.span_len[1] + 1))
        ln = min(ln, T)
        st = int(r.integers(0, T - ln + 1))
        sh = float(r.uniform(w.span_shift[0], w.span_shift[1])) if w.span_shift[0] != w.span_shift[1] \
            else float(w.span_shift[0])
        out[i] = (st, st + ln, sh)
    return out


def span_shift_profile(w: Workload, b: int, T: int) -> np.ndarray:
    """[T] shift magnitude per position (0 outside spans; first span covering a position wins)."""
    prof = np.zeros(T, np.float32)
    for st, en, sh in spans(w, b, T):
        seg = prof[int(st):int(en)]
        seg[seg == 0] = sh
    return prof


def unit_q(w: Workload, l: int, b: int, h: int, event: int = 0) -> np.ndarray:
    """Query window of one unit, [G, W, D] in storage dtype."""
    x = _rng(w.seed, _Q_STREAM, l, b, h, event).standard_normal((w.G, w.W, w.D), dtype=np.float32)
    return _store(x, w.dtype)


def unit_kv(w: Workload, l: int, b: int, h: int, T: int, q0: Optional[np.ndarray] = None,
            prof: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Initial cache of one unit: K, V [T, D] in storage dtype, spans planted against q0
    (the unit's event-0 query window; drawn here when not given)."""
    k = _rng(w.seed, _K_STREAM, l, b, h, 0).standard_normal((T, w.D), dtype=np.float32)
    v = _rng(w.seed, _V_STREAM, l, b, h, 0).standard_normal((T, w.D), dtype=np.float32)
    if w.n_spans > 0:
        if q0 is None:
            q0 = unit_q(w, l, b, h, 0)
        if prof is None:
            prof = span_shift_profile(w, b, T)
        qbar = as_f32(q0).reshape(-1, w.D).astype(np.float64).mean(axis=0)
        qdir = (qbar / np.linalg.norm(qbar)).astype(np.float32)
        k += prof[:, None] * qdir[None, :]
    return _store(k, w.dtype), _store(v, w.dtype)


def unit_fresh_rows(w: Workload, l: int, b: int, h: int, event: int, n: int) -> Tuple[np.ndarray, np.ndarray]:
    """n freshly decoded rows appended before compression event `event` (>= 1): plain N(0,1)."""
    k = _rng(w.seed, _K_STREAM, l, b, h, event).standard_normal((n, w.D), dtype=np.float32)
    v = _rng(w.seed, _V_STREAM, l, b, h, event).standard_normal((n, w.D), dtype=np.float32)
    return _store(k, w.dtype), _store(v, w.dtype)


def unit_ids(w: Workload) -> Sequence[Tuple[int, int, int]]:
    return [(l, b, h) for l in range(w.L) for b in range(w.B) for h in range(w.H)]


def dense_cache(w: Workload, n_threads: int = 8, t_capacity: Optional[int] = None):
    """Whole dense cache of a workload on the host.

    Returns dict(Q [L,B,H*G,W,D], K, V [L,B,H,Tcap,D], seq_lens [B]) in storage dtype
    (float32, or uint16 holding bf16 bits).  Rows beyond a sequence's length are zero.
    """
    lens = seq_lens(w)
    tcap = int(t_capacity or w.T)
    st = np.float32 if w.dtype == "f32" else np.uint16
    Q = np.zeros((w.L, w.B, w.H * w.G, w.W, w.D), st)
    K = np.zeros((w.L, w.B, w.H, tcap, w.D), st)
    V = np.zeros((w.L, w.B, w.H, tcap, w.D), st)
    profs = [span_shift_profile(w, b, int(lens[b])) if w.n_spans > 0 else None for b in range(w.B)]

    def fill(u):
        l, b, h = u
        T = int(lens[b])
        q = unit_q(w, l, b, h, 0)
        Q[l, b, h * w.G:(h + 1) * w.G] = q
        k, v = unit_kv(w, l, b, h, T, q, profs[b])
        K[l, b, h, :T] = k
        V[l, b, h, :T] = v

    with ThreadPoolExecutor(max_workers=n_threads) as ex:
        list(ex.map(fill, unit_ids(w)))
    return dict(Q=Q, K=K, V=V, seq_lens=lens)


def block_tables(w: Workload, lens: np.ndarray, kept_rows: int):
    """Paged layout bookkeeping: random physical placement of every sequence's source blocks and
    fresh destination blocks for `kept_rows` compact rows per sequence.

    Returns (src_table [B, max_blocks], dst_table [B, dst_blocks], n_slots); unused entries are -1.
    """
    blk = w.block
    nb = [(int(t) + blk - 1) // blk for t in lens]
    max_blocks = max(nb)
    dst_blocks = (kept_rows + blk - 1) // blk
    total = sum(nb) + w.B * dst_blocks
    perm = _rng(w.seed, _TABLE_STREAM).permutation(total).astype(np.int32)
    src = np.full((w.B, max_blocks), -1, np.int32)
    dst = np.full((w.B, dst_blocks), -1, np.int32)
    o = 0
    for b in range(w.B):
        src[b, :nb[b]] = perm[o:o + nb[b]]
        o += nb[b]
    for b in range(w.B):
        dst[b] = perm[o:o + dst_blocks]
        o += dst_blocks
    return src, dst, total * blk


def paged_pool_from_dense(w: Workload, X: np.ndarray, lens: np.ndarray, src_table: np.ndarray,
                          n_slots: int) -> np.ndarray:
    """Scatters a dense [L,B,H,Tcap,D] tensor into per-layer pools [L, slots, H, D]."""
    L, B, H, _, D = X.shape
    pool = np.zeros((L, n_slots, H, D), X.dtype)
    blk = w.block
    for b in range(B):
        T = int(lens[b])
        p = np.arange(T)
        slots = src_table[b, p // blk].astype(np.int64) * blk + p % blk
        for l in range(L):
            pool[l, slots] = np.transpose(X[l, b, :, :T], (1, 0, 2))
    return pool
