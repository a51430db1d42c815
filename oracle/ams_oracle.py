"""ctypes front end of the CPU oracle (oracle/ams_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  Takes and returns numpy arrays; bf16 inputs are
passed as uint16 and widened exactly to float32 here (a shift, no rounding).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

SCORER_LAST_QUERY, SCORER_MEAN_WINDOW, SCORER_KEYDIFF, SCORER_EXPECTED = 0, 1, 2, 3
SCORER_EXPECTED_VNORM = 5
SCORER_REDUNDANCY = 6

_lib = None


class _UnitParams(C.Structure):
    _fields_ = [("G", C.c_int), ("W", C.c_int), ("T", C.c_int), ("D", C.c_int),
                ("scorer", C.c_int), ("budget", C.c_int), ("S", C.c_int), ("q_min", C.c_int),
                ("lam", C.c_float), ("beta", C.c_float), ("eps", C.c_float),
                ("n_sink", C.c_int), ("n_last", C.c_int), ("causal", C.c_int),
                ("delta", C.c_float), ("l_min", C.c_int), ("l_max", C.c_int), ("pool_kernel", C.c_int),
                ("vnorm_eps", C.c_float), ("mix_lambda", C.c_float), ("score_kernel", C.c_int)]


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        _lib.amso_compress_many.restype = C.c_int
    return _lib


def widen(x: np.ndarray) -> np.ndarray:
    """float32 view of the values: uint16 arrays hold bf16 bit patterns."""
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32)
    return np.ascontiguousarray(x, dtype=np.float32)


def _f(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _i(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def score(Q, K, G, W, scorer=SCORER_MEAN_WINDOW, causal=False):
    """Q [G*W, D], K [T, D] -> (u [T], g [T]) float32."""
    Q = np.ascontiguousarray(widen(Q)).reshape(G * W, -1)
    K = np.ascontiguousarray(widen(K))
    T, D = K.shape
    assert Q.shape == (G * W, D)
    u = np.empty(T, np.float32)
    g = np.empty(T, np.float32)
    _chk(lib().amso_score(_f(Q), _f(K), G, W, T, D, int(scorer), int(bool(causal)), _f(u), _f(g)), "score")
    return u, g


def value_weight(e, V, eps=1e-2):
    """(softmax(e) + eps) * row norms of V."""
    e = np.ascontiguousarray(e, np.float32)
    V = np.ascontiguousarray(widen(V))
    g = np.empty_like(e)
    _chk(lib().amso_value_weight(_f(e), _f(V), V.shape[0], V.shape[1], C.c_float(eps), _f(g)), "value_weight")
    return g


def redundancy_score(u, K, mix_lambda=0.07, kernel=7):
    """u [T], K [T, D] (float32 or bf16 bits) -> g [T]: mix_lambda * pooled u - (1 - mix_lambda) * softmax of the
    mean cosine similarity of a key to the other keys."""
    Kf = np.ascontiguousarray(widen(K))
    u = np.ascontiguousarray(u, dtype=np.float32)
    T, D = Kf.shape
    g = np.empty(T, np.float32)
    _chk(lib().amso_redundancy_score(_f(u), _f(Kf), T, D, C.c_float(mix_lambda), int(kernel), _f(g)), "redundancy_score")
    return g


def mass(u, eps=1e-6):
    u = np.ascontiguousarray(u, np.float32)
    m = np.empty_like(u)
    _chk(lib().amso_mass(_f(u), len(u), C.c_float(eps), _f(m)), "mass")
    return m


def ema(m_cur, credit, lam, beta):
    """Returns (m_used, new_credit); the caller's credit array is not modified."""
    m_cur = np.ascontiguousarray(m_cur, np.float32)
    c = np.array(credit, dtype=np.float32, copy=True)
    out = np.empty_like(m_cur)
    _chk(lib().amso_ema(_f(m_cur), _f(c), len(m_cur), C.c_float(lam), C.c_float(beta), _f(out)), "ema")
    return out, c


def segment(m_used, S):
    m_used = np.ascontiguousarray(m_used, np.float32)
    bounds = np.empty(S + 1, np.int32)
    seg_mass = np.empty(S, np.float32)
    _chk(lib().amso_segment(_f(m_used), len(m_used), S, _i(bounds), _f(seg_mass)), "segment")
    return bounds, seg_mass


def pool(u, kernel):
    u = np.ascontiguousarray(u, np.float32)
    out = np.empty_like(u)
    _chk(lib().amso_pool(_f(u), len(u), int(kernel), _f(out)), "pool")
    return out


def segment_adaptive(m_used, delta, l_min, l_max, cap):
    """-> (bounds [cap+1], seg_mass [cap], n_seg)."""
    m_used = np.ascontiguousarray(m_used, np.float32)
    bounds = np.empty(cap + 1, np.int32)
    seg_mass = np.empty(cap, np.float32)
    n = C.c_int32(0)
    _chk(lib().amso_segment_adaptive(_f(m_used), len(m_used), C.c_float(delta), int(l_min), int(l_max), int(cap),
                                     _i(bounds), _f(seg_mass), C.byref(n)), "segment_adaptive")
    return bounds, seg_mass, n.value


def quota(bounds, seg_mass, budget, q_min=1):
    bounds = np.ascontiguousarray(bounds, np.int32)
    seg_mass = np.ascontiguousarray(seg_mass, np.float32)
    S = len(seg_mass)
    q = np.empty(S, np.int32)
    _chk(lib().amso_quota(_i(bounds), _f(seg_mass), S, int(budget), int(q_min), _i(q)), "quota")
    return q


def select(g, bounds, quota_):
    g = np.ascontiguousarray(g, np.float32)
    bounds = np.ascontiguousarray(bounds, np.int32)
    quota_ = np.ascontiguousarray(quota_, np.int32)
    idx = np.empty(max(int(quota_.sum()), 1), np.int32)
    n = C.c_int32(0)
    _chk(lib().amso_select(_f(g), _i(bounds), _i(quota_), len(quota_), _i(idx), C.byref(n)), "select")
    return idx[: n.value].copy()


def must_keep(T, budget, n_sink, n_last):
    """-> (sink_eff, last_eff, seg_budget)."""
    a, b, c = C.c_int(0), C.c_int(0), C.c_int(0)
    _chk(lib().amso_must_keep(int(T), int(budget), int(n_sink), int(n_last), C.byref(a), C.byref(b), C.byref(c)),
         "must_keep")
    return a.value, b.value, c.value


def finalize(g, seg_idx, sink_eff, last_eff, target):
    """Union with the must-keep positions, dedupe, sort, trim / backfill to target."""
    g = np.ascontiguousarray(g, np.float32)
    seg_idx = np.ascontiguousarray(seg_idx, np.int32)
    idx = np.empty(max(int(target), 1), np.int32)
    n = C.c_int32(0)
    _chk(lib().amso_finalize(_f(g), len(g), _i(seg_idx), len(seg_idx), int(sink_eff), int(last_eff), int(target),
                             _i(idx), C.byref(n)), "finalize")
    return idx[: n.value].copy()


def compact(K, V, credit, idx):
    """Row gather of K, V ([T, ...] any dtype) and credit [T]."""
    K = np.ascontiguousarray(K)
    V = np.ascontiguousarray(V)
    idx = np.ascontiguousarray(idx, np.int32)
    row_bytes = K[0].nbytes
    Ko = np.zeros((len(idx),) + K.shape[1:], K.dtype)
    Vo = np.zeros((len(idx),) + V.shape[1:], V.dtype)
    c = np.ascontiguousarray(credit, np.float32)
    co = np.zeros(len(idx), np.float32)
    _chk(lib().amso_compact(K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p), _f(c),
                            C.c_int64(row_bytes), _i(idx), len(idx),
                            Ko.ctypes.data_as(C.c_void_p), Vo.ctypes.data_as(C.c_void_p), _f(co)),
         "compact")
    return Ko, Vo, co


def compact_paged(K_pool, V_pool, src_table, K_pool_out, V_pool_out, dst_table, block, h, idx):
    """Pools are [slots, H, D]; writes rows of head h into the *_out pools in place."""
    H = K_pool.shape[1]
    row_bytes = K_pool[0, 0].nbytes
    src_table = np.ascontiguousarray(src_table, np.int32)
    dst_table = np.ascontiguousarray(dst_table, np.int32)
    idx = np.ascontiguousarray(idx, np.int32)
    for a in (K_pool, V_pool, K_pool_out, V_pool_out):
        assert a.flags["C_CONTIGUOUS"]
    _chk(lib().amso_compact_paged(K_pool.ctypes.data_as(C.c_void_p), V_pool.ctypes.data_as(C.c_void_p),
                                  _i(src_table), K_pool_out.ctypes.data_as(C.c_void_p),
                                  V_pool_out.ctypes.data_as(C.c_void_p), _i(dst_table),
                                  int(block), int(H), int(h), C.c_int64(row_bytes), _i(idx), len(idx)),
         "compact_paged")


def compress_unit(Q, K, V, credit, *, G, W, budget, S, lam, beta=0.9, eps=1e-6, q_min=1,
                  scorer=SCORER_MEAN_WINDOW, n_sink=0, n_last=0, causal=False, delta=0.0, l_min=0, l_max=0,
                  pool_kernel=0, vnorm_eps=1e-2, mix_lambda=0.07, score_kernel=7):
    """One whole event for one unit.  K, V [T, D] in storage dtype (float32 or
    uint16 = bf16 bits).  Returns a dict with every intermediate."""
    Kf = np.ascontiguousarray(widen(K))
    Qf = np.ascontiguousarray(widen(Q)).reshape(G * W, -1)
    K = np.ascontiguousarray(K)
    V = np.ascontiguousarray(V)
    T, D = Kf.shape
    kept = min(budget, T)
    p = _UnitParams(G, W, T, D, int(scorer), int(budget), int(S), int(q_min), lam, beta, eps,
                    int(n_sink), int(n_last), int(bool(causal)), delta, int(l_min), int(l_max), int(pool_kernel),
                    vnorm_eps, mix_lambda, int(score_kernel))
    Vf = np.ascontiguousarray(widen(V)) if int(scorer) == SCORER_EXPECTED_VNORM else None
    c = np.array(credit, dtype=np.float32, copy=True)
    out = dict(u=np.empty(T, np.float32), g=np.empty(T, np.float32), m_used=np.empty(T, np.float32),
               bounds=np.empty(S + 1, np.int32), seg_mass=np.empty(S, np.float32),
               quota=np.empty(S, np.int32), idx=np.full(kept, -1, np.int32),
               K_out=np.zeros((kept, D), K.dtype), V_out=np.zeros((kept, D), V.dtype),
               credit_out=np.zeros(kept, np.float32))
    n = C.c_int32(0)
    _chk(lib().amso_compress_unit(
        C.byref(p), _f(Qf), _f(Kf), _f(Vf) if Vf is not None else None,
        K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p),
        C.c_int64(K[0].nbytes), _f(c), _f(out["u"]), _f(out["g"]), _f(out["m_used"]),
        _i(out["bounds"]), _f(out["seg_mass"]), _i(out["quota"]), _i(out["idx"]), C.byref(n),
        out["K_out"].ctypes.data_as(C.c_void_p), out["V_out"].ctypes.data_as(C.c_void_p),
        _f(out["credit_out"])), "compress_unit")
    out["n_kept"] = n.value
    out["credit"] = c
    return out


def compress_many(Q, K, credit, *, G, W, budget, S, lam, beta=0.9, eps=1e-6, q_min=1,
                  scorer=SCORER_MEAN_WINDOW, n_threads=0, want_scores=False, K_rows=None, V_rows=None,
                  n_sink=0, n_last=0, causal=False, delta=0.0, l_min=0, l_max=0, pool_kernel=0, vnorm_eps=1e-2,
                  V=None, mix_lambda=0.07, score_kernel=7):
    """Q [U, G*W, D], K [U, T, D] float32 (already widened), credit [U, T] (updated in
    place).  K_rows, V_rows [U, T, D] in the storage dtype: when given, the kept rows are
    gathered as well (whole event).  Returns (idx [U, budget], n_kept [U], threads_used[, u, g])."""
    U, T, D = K.shape
    assert Q.shape == (U, G * W, D) and credit.shape == (U, T)
    for a in (Q, K, credit):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    p = _UnitParams(G, W, T, D, int(scorer), int(budget), int(S), int(q_min), lam, beta, eps,
                    int(n_sink), int(n_last), int(bool(causal)), delta, int(l_min), int(l_max), int(pool_kernel),
                    vnorm_eps, mix_lambda, int(score_kernel))
    if int(scorer) == SCORER_EXPECTED_VNORM:
        assert V is not None and V.shape == K.shape and V.dtype == np.float32 and V.flags["C_CONTIGUOUS"]
    idx = np.empty((U, budget), np.int32)
    n_kept = np.empty(U, np.int32)
    u = np.empty((U, T), np.float32) if want_scores else None
    g = np.empty((U, T), np.float32) if want_scores else None
    gather = K_rows is not None and V_rows is not None
    if gather:
        assert K_rows.shape == (U, T, D) and K_rows.flags["C_CONTIGUOUS"] and V_rows.flags["C_CONTIGUOUS"]
        K_out = np.zeros((U, budget, D), K_rows.dtype)
        V_out = np.zeros((U, budget, D), V_rows.dtype)
        c_out = np.zeros((U, budget), np.float32)
    vp = lambda a: a.ctypes.data_as(C.c_void_p)
    rc = lib().amso_compress_many(C.byref(p), U, int(n_threads), _f(Q), C.c_int64(G * W * D), _f(K),
                                  C.c_int64(T * D), _f(V) if V is not None else None, _f(credit), C.c_int64(T),
                                  _f(u) if want_scores else None, _f(g) if want_scores else None,
                                  _i(idx), _i(n_kept),
                                  vp(K_rows) if gather else None, vp(V_rows) if gather else None,
                                  C.c_int64(K_rows[0, 0].nbytes if gather else 0),
                                  vp(K_out) if gather else None, vp(V_out) if gather else None,
                                  _f(c_out) if gather else None)
    if rc <= 0:
        raise RuntimeError(f"oracle compress_many failed with code {rc}")
    return (idx, n_kept, rc, u, g) if want_scores else (idx, n_kept, rc)
