"""The entry point that allocates nothing (ams_mass_segment_static: scratch in the library's own device
array) against ams_mass_segment with a caller's workspace, through the C ABI: two calls in a row, the
second on a smaller input, bounds bit-exact and segment masses bit-exact (same kernels, same order)."""
import numpy as np
import pytest
import torch

from paper_2605_23200_amd import binding as B
from gpu_util import DEV, workspace

pytestmark = pytest.mark.gpu


def _case(units_shape, T, S, seed, delta=0.0, l_min=0, l_max=0):
    L, Bt, H = units_shape
    p = B.make_params(n_layers=L, batch=Bt, n_kv_heads=H, group=1, window=8, t_max=T, budget=min(256, T),
                      n_segments=S, seg_delta=delta, l_min=l_min, l_max=l_max)
    rng = np.random.default_rng(seed)
    lens = rng.integers(max(1, T // 3), T + 1, size=Bt).astype(np.int32)
    lens[0] = T
    m = rng.random((p.units, T), dtype=np.float32) ** 4
    for i in range(p.units):
        t = int(lens[(i // H) % Bt])
        m[i, :t] /= m[i, :t].astype(np.float64).sum()
    return p, torch.from_numpy(lens).to(DEV), torch.from_numpy(m).to(DEV)


def _run(p, lens, m, static):
    bounds = torch.full((p.units, p.n_segments + 1), -5, dtype=torch.int32, device=DEV)
    mass = torch.full((p.units, p.n_segments), -5.0, dtype=torch.float32, device=DEV)
    if static:
        B.ams_mass_segment_static(p, lens, m, bounds, mass)
    else:
        B.ams_mass_segment(p, lens, m, bounds, mass, workspace(p))
    torch.cuda.synchronize()
    return bounds.cpu().numpy(), mass.cpu().numpy()


def test_static_scratch_entry_matches_the_workspace_entry():
    big = _case((2, 3, 4), 20000, 16, seed=11)            # 24 units, 5 chunks each, ragged lengths
    small = _case((1, 2, 2), 3000, 8, seed=12)            # then a smaller problem: stale scratch must not matter
    delta = _case((1, 1, 3), 9000, 10 + 1 + 9000 // 256, seed=13, delta=0.1, l_min=16, l_max=256)
    for p, lens, m in (big, small, delta, big):
        b_ws, m_ws = _run(p, lens, m, static=False)
        b_st, m_st = _run(p, lens, m, static=True)
        np.testing.assert_array_equal(b_st, b_ws)
        np.testing.assert_array_equal(m_st.view(np.uint32), m_ws.view(np.uint32))
        assert (b_st[:, 0] == 0).all() and (np.diff(b_st, axis=1) >= 0).all()


def test_static_scratch_entry_rejects_what_does_not_fit():
    p = B.make_params(n_layers=64, batch=16, n_kv_heads=8, group=1, window=8, t_max=131072, budget=256, n_segments=64)
    assert p.units * 32 * 8 > (1 << 20)                   # the chunk totals alone exceed the array
    rc = B.lib().ams_mass_segment_static(B.C.byref(p), 64, 64, 64, 64, None)
    assert rc == B.ERR_UNSUPPORTED
