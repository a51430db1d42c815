"""Helpers shared by the GPU parity tests: upload of synthetic caches, oracle calls per unit."""
import numpy as np
import torch

from paper_2605_23200_amd import binding as B
from paper_2605_23200_amd import inputs

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Host array -> device tensor with the same bytes (bf16 bit patterns travel as int16)."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host(t: torch.Tensor, like_dtype=None) -> np.ndarray:
    a = t.detach().cpu().numpy()
    if like_dtype == np.uint16:
        a = a.view(np.uint16)
    return a


def params_for(w: inputs.Workload, scorer=B.SCORER_MEAN_WINDOW, t_stride=None, **over):
    kw = dict(n_layers=w.L, batch=w.B, n_kv_heads=w.H, group=w.G, window=w.W, head_dim=w.D,
              kv_dtype=B.F32 if w.dtype == "f32" else B.BF16, t_max=w.T, t_stride=t_stride or w.T,
              budget=w.budget, n_segments=w.S, q_min=w.q_min, ema_lambda=w.lam, ema_beta=w.beta,
              mass_eps=w.eps, scorer=scorer, n_sink=w.n_sink, n_last=w.n_last, causal=w.causal,
              seg_delta=w.seg_delta, l_min=w.l_min, l_max=w.l_max, pool_kernel=w.pool_kernel)
    kw.update(over)
    return B.make_params(**kw)


def workspace(p) -> torch.Tensor:
    n = B.ams_workspace_bytes(p)
    assert n > 0
    return torch.zeros(n, dtype=torch.uint8, device=DEV)


def unit_list(w):
    return inputs.unit_ids(w)


def assert_close_rel(got, want, rtol=1e-5, atol=1e-12, what=""):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    err = np.abs(got - want)
    tol = atol + rtol * np.abs(want)
    bad = err > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} beyond rtol={rtol}; worst rel "
                           f"{(err / np.maximum(np.abs(want), 1e-300)).max():.3e} at {np.argmax(err / np.maximum(tol, 1e-300))}")


def score_term_magnitudes(scorer, Q, K):
    """Per key, the sum of the magnitudes of the terms that the signed base scores add up (what a relative bound
    has to be relative to when the sum itself passes through zero).  Q [N, D], K [T, D], float32 or bf16 bits.
    KeyDiff (-cos(k_t, kbar)): sum_d |k_td kbar_d| / (|k_t| |kbar|).
    Expected attention (mu.k/sqrt(D) + k'Sigma k/(2D)): sum_d |mu_d k_td| / sqrt(D) plus the quadratic form, which
    is a variance and cannot cancel."""
    widen = lambda x: (inputs.bf16_bits_to_f32(x) if x.dtype == np.uint16 else x).astype(np.float64)
    K = widen(np.asarray(K))
    D = K.shape[1]
    if scorer == B.SCORER_KEYDIFF:
        kbar = K.mean(axis=0)
        den = np.linalg.norm(K, axis=1) * np.linalg.norm(kbar)
        return np.where(den > 0, (np.abs(K) @ np.abs(kbar)) / np.maximum(den, 1e-300), 0.0)
    if scorer == B.SCORER_EXPECTED:
        Q = widen(np.asarray(Q)).reshape(-1, D)
        mu = Q.mean(axis=0)
        s = (Q - mu) @ K.T / np.sqrt(D)
        return (np.abs(K) @ np.abs(mu)) / np.sqrt(D) + 0.5 * (s * s).mean(axis=0)
    raise ValueError(scorer)


def assert_close_terms(got, want, magnitude, rtol=1e-5, atol=1e-12, what=""):
    """For results that are a signed sum of terms (and may pass through zero): the error of every element is
    held against rtol times the sum of the magnitudes of ITS terms (`magnitude`, same shape), not against the
    vector's largest value."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    err = np.abs(got - want)
    tol = atol + rtol * np.asarray(magnitude, np.float64)
    bad = err > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} beyond rtol={rtol} of their terms; worst ratio "
                           f"{(err / np.maximum(tol, 1e-300)).max():.3f} at {np.argmax(err / np.maximum(tol, 1e-300))}")
