"""The C-ABI library loads and exports every symbol include/ams.h declares; argument errors are
reported by status on the host, without a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2605_23200_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ams.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ams_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert B.status_string(0) == "ok"
    assert "workspace" in B.status_string(B.ERR_WORKSPACE_TOO_SMALL)


def _good():
    return B.make_params(n_layers=2, batch=1, n_kv_heads=8, group=4, window=32, t_max=4096, budget=512,
                         n_segments=8)


def test_workspace_bytes_and_layout():
    p = _good()
    n = B.ams_workspace_bytes(p)
    assert n >= 3 * p.units * p.t_stride * 4
    lay = B.ams_workspace_layout(p)
    assert lay.u == lay.g and lay.m_used > lay.u and lay.quota < n
    p.scorer = B.SCORER_EXPECTED
    lay = B.ams_workspace_layout(p)
    assert lay.u != lay.g


@pytest.mark.parametrize("field,value,status", [
    ("budget", 0, B.ERR_INVALID_ARG), ("n_segments", 0, B.ERR_INVALID_ARG), ("t_stride", 100, B.ERR_INVALID_ARG),
    ("ema_lambda", 1.0, B.ERR_INVALID_ARG), ("ema_lambda", -0.1, B.ERR_INVALID_ARG),
    ("ema_beta", 1.5, B.ERR_INVALID_ARG), ("mass_eps", 0.0, B.ERR_INVALID_ARG), ("kv_dtype", 7, B.ERR_INVALID_ARG),
    ("scorer", 9, B.ERR_INVALID_ARG), ("head_dim", 96, B.ERR_UNSUPPORTED), ("n_segments", 5000, B.ERR_UNSUPPORTED),
    ("window", 100, B.ERR_UNSUPPORTED), ("n_layers", 10000, B.ERR_UNSUPPORTED),
    ("n_sink", -1, B.ERR_INVALID_ARG), ("n_last", -3, B.ERR_INVALID_ARG), ("causal", 2, B.ERR_INVALID_ARG),
    ("pool_kernel", 4, B.ERR_INVALID_ARG), ("pool_kernel", 65, B.ERR_INVALID_ARG), ("seg_delta", -0.1, B.ERR_INVALID_ARG),
    ("seg_delta", 1e-4, B.ERR_INVALID_ARG),            # more than 1024 initial segments
    ("seg_delta", 0.05, B.ERR_INVALID_ARG),            # 20 initial segments do not fit the 8 entries
    ("l_max", 64, B.ERR_INVALID_ARG),                  # length rules without a target mass
    ("score_path", 4, B.ERR_INVALID_ARG), ("score_path", -1, B.ERR_INVALID_ARG),
    ("scorer", 7, B.ERR_INVALID_ARG)])
def test_bad_params_are_rejected_on_the_host(field, value, status):
    p = _good()
    setattr(p, field, value)
    assert B.ams_workspace_bytes(p) == 0
    out = B.WorkspaceView()
    assert B.lib().ams_workspace_layout(C.byref(p), C.byref(out)) == status
    # the launching entry points return the same status before touching any pointer
    assert B.lib().ams_ema_update(C.byref(p), None, None, None, None, None, 0, None) == status


def test_score_path_field():
    p = _good()
    for path in (B.SCORE_PATH_AUTO, B.SCORE_PATH_TWO_SWEEPS, B.SCORE_PATH_ONE_READ, B.SCORE_PATH_ONE_LAUNCH):
        p.score_path = path
        assert B.ams_workspace_bytes(p) > 0            # the workspace does not depend on the path


def test_redundancy_scorer_parameters():
    p = _good()
    p.scorer = B.SCORER_REDUNDANCY
    assert B.ams_workspace_bytes(p) > 0                # defaults: lambda 0.07, kernel 7
    for field, bad in (("mix_lambda", 1.5), ("mix_lambda", -0.1), ("score_kernel", 4), ("score_kernel", 65),
                       ("score_kernel", -1)):
        q = _good()
        q.scorer = B.SCORER_REDUNDANCY
        setattr(q, field, bad)
        assert B.ams_workspace_bytes(q) == 0
    q = _good()
    q.mix_lambda = 7.0                                 # ignored by the other scorers
    assert B.ams_workspace_bytes(q) > 0


def test_both_head_dimensions_are_accepted():
    p = _good()
    for d in (64, 128):
        p.head_dim = d
        assert B.ams_workspace_bytes(p) > 0


def test_segmentation_capacity_rule():
    # target mass 0.1 -> 10 initial segments; with L_max = 256 up to 4096 / 256 = 16 more
    p = _good()
    p.seg_delta, p.l_min, p.l_max = 0.1, 16, 256
    p.n_segments = 25
    assert B.ams_workspace_bytes(p) == 0
    p.n_segments = 26
    assert B.ams_workspace_bytes(p) > 0
    p.l_min = 300                                      # L_min above L_max
    assert B.ams_workspace_bytes(p) == 0


def test_optional_features_need_their_inputs():
    L = B.lib()
    p = _good()
    p.n_sink = 4                                       # the must-keep path needs the workspace
    assert L.ams_select(C.byref(p), 64, 64, 64, 64, 64, 64, 64, None, 0, None) == B.ERR_INVALID_ARG
    assert L.ams_select(C.byref(p), 64, 64, 64, 64, 64, 64, 64, 64, 16, None) == B.ERR_WORKSPACE_TOO_SMALL
    p = _good()
    p.scorer = B.SCORER_EXPECTED_VNORM                 # the value-weighted scorer needs V
    v = B.KvView(B.LAYOUT_DENSE, 64, None, 4096, None, 0, 0, 0)
    assert L.ams_score(C.byref(p), C.byref(v), 64, 64, 64, 64, 64, 1 << 40, None) == B.ERR_INVALID_ARG
    p.vnorm_eps = -1.0
    assert B.ams_workspace_bytes(p) == 0


def test_null_pointers_are_rejected_without_launch():
    p = _good()
    L = B.lib()
    assert L.ams_ema_update(C.byref(p), None, None, None, None, None, 0, None) == B.ERR_INVALID_ARG
    assert L.ams_mass_segment(C.byref(p), None, None, None, None, None, 0, None) == B.ERR_INVALID_ARG
    assert L.ams_select(C.byref(p), None, None, None, None, None, None, None, None, 0, None) == B.ERR_INVALID_ARG
    v = B.KvView(B.LAYOUT_DENSE, None, None, 4096, None, 0, 0, 0)
    assert L.ams_score(C.byref(p), C.byref(v), None, None, None, None, None, 0, None) == B.ERR_INVALID_ARG
    v = B.KvView(B.LAYOUT_PAGED, 64, 64, 0, 64, 1000, 32, 100000)     # block size 32
    assert L.ams_compact(C.byref(p), C.byref(v), None, None, C.byref(v), None, None, None) == B.ERR_UNSUPPORTED
    v = B.KvView(B.LAYOUT_DENSE, 64, 64, 100, None, 0, 0, 0)          # capacity below t_max
    assert L.ams_compact(C.byref(p), C.byref(v), None, None, C.byref(v), None, None, None) == B.ERR_INVALID_ARG
    assert L.ams_workspace_bytes(None) == 0
