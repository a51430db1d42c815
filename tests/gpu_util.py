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


def assert_close_norm(got, want, rtol=1e-5, what=""):
    """For signed scores that pass through zero: error relative to the largest magnitude of the vector."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    scale = np.abs(want).max()
    err = np.abs(got - want).max()
    assert err <= rtol * scale, f"{what}: max abs err {err:.3e} vs scale {scale:.3e} (ratio {err / scale:.3e})"


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
