"""Device-side bookkeeping for running compression events on a synthetic workload.

Allocation and upload only (PyTorch is the allocator); every step of the method runs inside the
C-ABI library.  Used by the tests, the smoke check and the benchmark.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import inputs


def _dev(a: np.ndarray, device) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class Job:
    """One workload resident on the GPU: source cache, destination cache, credit, outputs, workspace."""

    def __init__(self, w: inputs.Workload, host: dict, scorer: int = B.SCORER_MEAN_WINDOW,
                 device: str = "cuda:0", credit: np.ndarray | None = None, paged: bool | None = None,
                 score_path: int = B.SCORE_PATH_AUTO):
        self.w, self.device = w, device
        lens = host["seq_lens"]
        self.t_max = int(lens.max())
        self.t_stride = (self.t_max + 63) // 64 * 64
        self.p = B.make_params(n_layers=w.L, batch=w.B, n_kv_heads=w.H, group=w.G, window=w.W,
                               head_dim=w.D, kv_dtype=B.F32 if w.dtype == "f32" else B.BF16,
                               t_max=self.t_max, t_stride=self.t_stride, budget=w.budget,
                               n_segments=w.S, q_min=w.q_min, ema_lambda=w.lam, ema_beta=w.beta,
                               mass_eps=w.eps, scorer=scorer, n_sink=w.n_sink, n_last=w.n_last,
                               causal=w.causal, seg_delta=w.seg_delta, l_min=w.l_min, l_max=w.l_max,
                               pool_kernel=w.pool_kernel, score_path=score_path)
        self.units = w.units
        self.keep = min(w.budget, self.t_max)
        self.lens = _dev(lens, device)
        self.Q = _dev(host["Q"], device)
        self.paged = w.paged if paged is None else paged
        if self.paged:
            self.src_table_h, self.dst_table_h, n_slots = inputs.block_tables(w, lens, self.keep)
            self.K = _dev(inputs.paged_pool_from_dense(w, host["K"], lens, self.src_table_h, n_slots), device)
            self.V = _dev(inputs.paged_pool_from_dense(w, host["V"], lens, self.src_table_h, n_slots), device)
            self.src_table, self.dst_table = _dev(self.src_table_h, device), _dev(self.dst_table_h, device)
            self.src = B.paged_view(self.K, self.V, self.src_table)
            # compaction writes into fresh blocks of the same pools
            self.dst = B.paged_view(self.K, self.V, self.dst_table)
            # the two views share base pointers on purpose; the library's aliasing check is for dense slabs
        else:
            # a caller that runs many jobs on one cache may upload it once and pass the device copies along
            self.K = host["K_dev"] if "K_dev" in host else _dev(host["K"], device)
            self.V = host["V_dev"] if "V_dev" in host else _dev(host["V"], device)
            self.Kd = torch.zeros((w.L, w.B, w.H, self.keep, w.D), dtype=self.K.dtype, device=device)
            self.Vd = torch.zeros_like(self.Kd)
            self.src = B.dense_view(self.K, self.V)
            self.dst = B.dense_view(self.Kd, self.Vd)
        self.credit = torch.zeros((self.units, self.t_stride), dtype=torch.float32, device=device)
        if credit is not None:
            self.credit[:, :credit.shape[1]] = torch.from_numpy(credit).to(device)
        self.credit_dst = torch.zeros((self.units, w.budget), dtype=torch.float32, device=device)
        self.idx = torch.full((self.units, w.budget), -9, dtype=torch.int32, device=device)
        self.n_kept = torch.zeros(self.units, dtype=torch.int32, device=device)
        self.ws = torch.zeros(B.ams_workspace_bytes(self.p), dtype=torch.uint8, device=device)

    def step(self, stream=None):
        B.ams_compress_step(self.p, self.src, self.lens, self.Q, self.credit, self.dst, self.credit_dst,
                            self.idx, self.n_kept, self.ws, stream)

    def set_queries(self, Q: np.ndarray):
        self.Q.copy_(_dev(Q, self.device))

    def intermediates(self) -> B.StepIntermediates:
        return B.workspace_tensors(self.p, self.ws)


class DeviceFilledPagedJob:
    """A paged, ragged workload too large to draw on the host (config 2: about 90 GB of pools): lengths and
    block tables come from the seeded generators of `inputs`, the K / V / Q VALUES are standard normal numbers
    drawn on the device (seeded), without planted spans.  For throughput runs only: there is no host copy to
    check against."""

    def __init__(self, w: inputs.Workload, scorer: int = B.SCORER_MEAN_WINDOW, device: str = "cuda:0", seed: int = 0):
        assert w.paged
        self.w, self.device, self.paged = w, device, True
        lens = inputs.seq_lens(w)
        self.lens_h = lens
        self.t_max = int(lens.max())
        self.t_stride = (self.t_max + 63) // 64 * 64
        self.keep = min(w.budget, self.t_max)
        self.units = w.units
        src, dst, n_slots = inputs.block_tables(w, lens, self.keep)
        dtype = torch.float32 if w.dtype == "f32" else torch.bfloat16
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.K = torch.empty((w.L, n_slots, w.H, w.D), dtype=dtype, device=device)
        self.V = torch.empty_like(self.K)
        for l in range(w.L):                       # layer by layer: no fp32 temporary of the whole pool
            self.K[l].normal_(generator=gen)
            self.V[l].normal_(generator=gen)
        self.Q = torch.randn((w.L, w.B, w.H * w.G, w.W, w.D), device=device, generator=gen).to(dtype)
        self.p = B.make_params(n_layers=w.L, batch=w.B, n_kv_heads=w.H, group=w.G, window=w.W, head_dim=w.D,
                               kv_dtype=B.F32 if w.dtype == "f32" else B.BF16, t_max=self.t_max,
                               t_stride=self.t_stride, budget=w.budget, n_segments=w.S, q_min=w.q_min,
                               ema_lambda=w.lam, ema_beta=w.beta, mass_eps=w.eps, scorer=scorer, n_sink=w.n_sink,
                               n_last=w.n_last, causal=w.causal, seg_delta=w.seg_delta, l_min=w.l_min,
                               l_max=w.l_max, pool_kernel=w.pool_kernel)
        self.lens = _dev(lens, device)
        self.src_table, self.dst_table = _dev(src, device), _dev(dst, device)
        self.src = B.paged_view(self.K, self.V, self.src_table)
        self.dst = B.paged_view(self.K, self.V, self.dst_table)
        self.credit = torch.zeros((self.units, self.t_stride), dtype=torch.float32, device=device)
        self.credit_dst = torch.zeros((self.units, w.budget), dtype=torch.float32, device=device)
        self.idx = torch.full((self.units, w.budget), -9, dtype=torch.int32, device=device)
        self.n_kept = torch.zeros(self.units, dtype=torch.int32, device=device)
        self.ws = torch.zeros(B.ams_workspace_bytes(self.p), dtype=torch.uint8, device=device)

    def step(self, stream=None):
        B.ams_compress_step(self.p, self.src, self.lens, self.Q, self.credit, self.dst, self.credit_dst,
                            self.idx, self.n_kept, self.ws, stream)

    def intermediates(self) -> B.StepIntermediates:
        return B.workspace_tensors(self.p, self.ws)
