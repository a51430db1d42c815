"""Thin Python face of the C-ABI library (include/ams.h): argument marshalling only.

Every function has the name and the argument order of its C entry point, takes torch tensors that
live on the GPU (PyTorch is used for device memory and streams, nothing else), passes their raw
pointers through ctypes and raises on a non-zero status.  There is no CPU fallback: if the built
library is missing, importing the entry points fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libams.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_HIP = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
SCORER_LAST_QUERY, SCORER_MEAN_WINDOW, SCORER_KEYDIFF, SCORER_EXPECTED, SCORER_EXTERNAL = 0, 1, 2, 3, 4
SCORER_EXPECTED_VNORM = 5
SCORER_REDUNDANCY = 6
LAYOUT_DENSE, LAYOUT_PAGED = 0, 1
SCORE_PATH_AUTO, SCORE_PATH_TWO_SWEEPS, SCORE_PATH_ONE_READ, SCORE_PATH_ONE_LAUNCH = 0, 1, 2, 3

EXPORTS = ("ams_status_string", "ams_workspace_bytes", "ams_workspace_layout", "ams_profile_begin",
           "ams_profile_end", "ams_debug_set_wait_limit", "ams_score",
           "ams_ema_update", "ams_mass_segment", "ams_mass_segment_static", "ams_select", "ams_compact",
           "ams_compress_step")


class AmsError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


class Params(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_kv_heads", C.c_int32),
                ("group", C.c_int32), ("head_dim", C.c_int32), ("window", C.c_int32),
                ("kv_dtype", C.c_int32), ("t_max", C.c_int32), ("t_stride", C.c_int64),
                ("budget", C.c_int32), ("n_segments", C.c_int32), ("q_min", C.c_int32),
                ("ema_lambda", C.c_float), ("ema_beta", C.c_float), ("mass_eps", C.c_float),
                ("scorer", C.c_int32), ("n_sink", C.c_int32), ("n_last", C.c_int32), ("causal", C.c_int32),
                ("seg_delta", C.c_float), ("l_min", C.c_int32), ("l_max", C.c_int32), ("pool_kernel", C.c_int32),
                ("vnorm_eps", C.c_float), ("score_path", C.c_int32),
                ("mix_lambda", C.c_float), ("score_kernel", C.c_int32)]

    @property
    def units(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads


class KvView(C.Structure):
    _fields_ = [("layout", C.c_int32), ("k", C.c_void_p), ("v", C.c_void_p), ("t_capacity", C.c_int64),
                ("block_table", C.c_void_p), ("max_blocks_per_seq", C.c_int32), ("block_size", C.c_int32),
                ("n_slots", C.c_int64)]


class WorkspaceView(C.Structure):
    _fields_ = [("u", C.c_size_t), ("g", C.c_size_t), ("m_used", C.c_size_t), ("bounds", C.c_size_t),
                ("seg_mass", C.c_size_t), ("quota", C.c_size_t)]


_lib = None


def lib() -> C.CDLL:
    """Loads the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2605_23200_amd.build` "
                              "(or __graft_entry__.build()) first")
        l = C.CDLL(LIB_PATH)
        l.ams_status_string.restype = C.c_char_p
        l.ams_status_string.argtypes = [C.c_int]
        l.ams_workspace_bytes.restype = C.c_size_t
        l.ams_workspace_bytes.argtypes = [C.POINTER(Params)]
        l.ams_workspace_layout.argtypes = [C.POINTER(Params), C.POINTER(WorkspaceView)]
        P, V, p = C.POINTER(Params), C.POINTER(KvView), C.c_void_p
        l.ams_score.argtypes = [P, V, p, p, p, p, p, C.c_size_t, p]
        l.ams_ema_update.argtypes = [P, p, p, p, p, p, C.c_size_t, p]
        l.ams_mass_segment.argtypes = [P, p, p, p, p, p, C.c_size_t, p]
        l.ams_mass_segment_static.argtypes = [P, p, p, p, p, p]
        l.ams_select.argtypes = [P, p, p, p, p, p, p, p, p, C.c_size_t, p]
        l.ams_compact.argtypes = [P, V, p, p, V, p, p, p]
        l.ams_compress_step.argtypes = [P, V, p, p, p, V, p, p, p, p, C.c_size_t, p]
        l.ams_profile_end.argtypes = [p, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_float)]
        for name in EXPORTS[2:]:
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().ams_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _check(rc: int, what: str):
    if rc != OK:
        raise AmsError(rc, what)


def make_params(*, n_layers, batch, n_kv_heads, group, window, head_dim=128, kv_dtype=BF16, t_max,
                t_stride=None, budget, n_segments, q_min=1, ema_lambda=0.9, ema_beta=0.9, mass_eps=1e-6,
                scorer=SCORER_MEAN_WINDOW, n_sink=0, n_last=0, causal=False, seg_delta=0.0, l_min=0, l_max=0,
                pool_kernel=0, vnorm_eps=1e-2, score_path=SCORE_PATH_AUTO,
                mix_lambda=0.07, score_kernel=7) -> Params:
    return Params(n_layers, batch, n_kv_heads, group, head_dim, window, kv_dtype, t_max,
                  t_stride if t_stride is not None else t_max, budget, n_segments, q_min,
                  ema_lambda, ema_beta, mass_eps, scorer, int(n_sink), int(n_last), int(bool(causal)),
                  float(seg_delta), int(l_min), int(l_max), int(pool_kernel), float(vnorm_eps), int(score_path),
                  float(mix_lambda), int(score_kernel))


def dense_view(k: torch.Tensor, v: Optional[torch.Tensor]) -> KvView:
    """k, v: [L, B, H, t_capacity, D] device tensors (any 2- or 4-byte element type)."""
    assert k.dim() == 5
    return KvView(LAYOUT_DENSE, k.data_ptr(), v.data_ptr() if v is not None else None, k.shape[3],
                  None, 0, 0, 0)


def paged_view(k_pool: torch.Tensor, v_pool: Optional[torch.Tensor], block_table: torch.Tensor,
               block_size: int = 16) -> KvView:
    """k_pool, v_pool: [L, n_slots, H, D]; block_table: int32 [B, max_blocks]."""
    assert k_pool.dim() == 4 and block_table.dtype == torch.int32 and block_table.is_contiguous()
    return KvView(LAYOUT_PAGED, k_pool.data_ptr(), v_pool.data_ptr() if v_pool is not None else None, 0,
                  block_table.data_ptr(), block_table.shape[1], block_size, k_pool.shape[1])


def ams_workspace_bytes(p: Params) -> int:
    return int(lib().ams_workspace_bytes(C.byref(p)))


def ams_workspace_layout(p: Params) -> WorkspaceView:
    out = WorkspaceView()
    _check(lib().ams_workspace_layout(C.byref(p), C.byref(out)), "ams_workspace_layout")
    return out


def ams_profile_begin():
    _check(lib().ams_profile_begin(), "ams_profile_begin")


def ams_debug_set_wait_limit(polls: int):
    _check(lib().ams_debug_set_wait_limit(int(polls)), "ams_debug_set_wait_limit")


def ams_profile_end(stream=None, max_entries: int = 4096):
    """Returns [(kernel label, milliseconds), ...] in launch order; waits for the stream."""
    labels = (C.c_char_p * max_entries)()
    ms = (C.c_float * max_entries)()
    n = lib().ams_profile_end(_stream(stream), max_entries, labels, ms)
    if n < 0:
        raise AmsError(-n, "ams_profile_end")
    return [(labels[i].decode(), float(ms[i])) for i in range(n)]


def ams_score(p, src, seq_lens, q, u, g, ws, stream=None):
    _check(lib().ams_score(C.byref(p), C.byref(src), _ptr(seq_lens), _ptr(q), _ptr(u), _ptr(g), _ptr(ws),
                           ws.numel() * ws.element_size(), _stream(stream)), "ams_score")


def ams_ema_update(p, seq_lens, u, credit, m_used, ws=None, stream=None):
    _check(lib().ams_ema_update(C.byref(p), _ptr(seq_lens), _ptr(u), _ptr(credit), _ptr(m_used), _ptr(ws),
                                ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "ams_ema_update")


def ams_mass_segment(p, seq_lens, m_used, bounds, seg_mass, ws=None, stream=None):
    _check(lib().ams_mass_segment(C.byref(p), _ptr(seq_lens), _ptr(m_used), _ptr(bounds), _ptr(seg_mass),
                                  _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                  _stream(stream)), "ams_mass_segment")


def ams_mass_segment_static(p, seq_lens, m_used, bounds, seg_mass, stream=None):
    _check(lib().ams_mass_segment_static(C.byref(p), _ptr(seq_lens), _ptr(m_used), _ptr(bounds), _ptr(seg_mass),
                                         _stream(stream)), "ams_mass_segment_static")


def ams_select(p, seq_lens, g, bounds, seg_mass, quota, idx, n_kept, ws=None, stream=None):
    _check(lib().ams_select(C.byref(p), _ptr(seq_lens), _ptr(g), _ptr(bounds), _ptr(seg_mass), _ptr(quota),
                            _ptr(idx), _ptr(n_kept), _ptr(ws),
                            ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "ams_select")


def ams_compact(p, src, idx, n_kept, dst, credit_src=None, credit_dst=None, stream=None):
    _check(lib().ams_compact(C.byref(p), C.byref(src), _ptr(idx), _ptr(n_kept), C.byref(dst),
                             _ptr(credit_src), _ptr(credit_dst), _stream(stream)), "ams_compact")


def ams_compress_step(p, src, seq_lens, q, credit, dst, credit_dst, idx, n_kept, ws, stream=None):
    _check(lib().ams_compress_step(C.byref(p), C.byref(src), _ptr(seq_lens), _ptr(q), _ptr(credit),
                                   C.byref(dst), _ptr(credit_dst), _ptr(idx), _ptr(n_kept), _ptr(ws),
                                   ws.numel() * ws.element_size(), _stream(stream)), "ams_compress_step")


@dataclass
class StepIntermediates:
    u: torch.Tensor
    g: torch.Tensor
    m_used: torch.Tensor
    bounds: torch.Tensor
    seg_mass: torch.Tensor
    quota: torch.Tensor


def workspace_tensors(p: Params, ws: torch.Tensor) -> StepIntermediates:
    """Typed views of the intermediates ams_compress_step left in `ws` (a uint8 device tensor)."""
    lay = ams_workspace_layout(p)
    U, S, ts = p.units, p.n_segments, p.t_stride

    def view(off, n, dtype, shape):
        return ws[off:off + n * 4].view(dtype).view(*shape)

    return StepIntermediates(
        u=view(lay.u, U * ts, torch.float32, (U, ts)), g=view(lay.g, U * ts, torch.float32, (U, ts)),
        m_used=view(lay.m_used, U * ts, torch.float32, (U, ts)),
        bounds=view(lay.bounds, U * (S + 1), torch.int32, (U, S + 1)),
        seg_mass=view(lay.seg_mass, U * S, torch.float32, (U, S)),
        quota=view(lay.quota, U * S, torch.int32, (U, S)))
