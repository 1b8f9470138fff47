"""The C-ABI library loads on a GPU-less host, exports every symbol the public
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2605_14978_amd as ppow
from paper_2605_14978_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ppow.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ppow_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"ppow_score_windows", "ppow_select_windows", "ppow_score_workspace_bytes",
            "ppow_select_workspace_bytes", "ppow_last_error", "ppow_version",
            "ppow_last_row_kernel", "ppow_adaw_sequence",
            "ppow_adaw_sequence_workspace_bytes", "ppow_score_windows_static", "ppow_release",
            "ppow_debug_cluster_wait_limit"} <= set(names)
    L = ppow.lib()
    for name in names:
        assert hasattr(L, name), f"{name} declared in ppow.h but not exported"


def test_struct_layouts_match_header():
    assert ctypes.sizeof(binding.PpowParams) == 28
    assert ctypes.sizeof(binding.PpowOutputs) == 18 * ctypes.sizeof(ctypes.c_void_p)


def test_workspace_queries():
    L = ppow.lib()
    scratch = 1 << 20
    assert L.ppow_score_workspace_bytes(16384, 8, 128256, binding.PPOW_BF16, 0) == scratch + 16384 * 8 * 32
    assert L.ppow_score_workspace_bytes(0, 8, 128256, binding.PPOW_BF16, 0) == scratch
    for bad in ((-1, 8, 100, 0), (4, 0, 100, 0), (4, 65, 100, 0), (4, 8, 1, 0), (4, 8, 100, 7),
                (1 << 30, 8, 100, 0), (4, 8, 1 << 31, 0)):
        assert L.ppow_score_workspace_bytes(*bad, 0) == 0
    assert L.ppow_select_workspace_bytes(65536, 8192) >= 256
    assert L.ppow_select_workspace_bytes(65536, 16384) == 16384 * 8
    for bad in ((0, 1), (10, 0), (10, 11), (1 << 31, 5)):
        assert L.ppow_select_workspace_bytes(*bad) == 0


def _score(L, *, draft=16, target=32, tokens=48, uniforms=64, B=4, K=2, V=100, dtype=0,
           params=None, outs=None, ws=4096, ws_bytes=1 << 24, null_params=False, null_outs=False):
    p = params or binding.PpowParams(0.05, 0.5, 1.0, 0, 0, 0, 0.0)
    o = outs or binding.PpowOutputs(*([4096] * 4 + [None] * 14))
    return L.ppow_score_windows(draft, target, tokens, uniforms, None, B, K, V, dtype,
                                None if null_params else ctypes.byref(p),
                                None if null_outs else ctypes.byref(o), ws, ws_bytes, None)


def test_score_argument_errors_return_before_any_launch():
    L = ppow.lib()
    E = binding.PPOW_ERR_INVALID_ARG
    assert _score(L, null_params=True) == E
    assert _score(L, null_outs=True) == E
    assert _score(L, B=-1) == E
    assert _score(L, K=0) == E
    assert _score(L, K=65) == E
    assert _score(L, V=1) == E
    assert _score(L, dtype=2) == E
    assert _score(L, draft=None) == E
    assert _score(L, target=None) == E
    assert _score(L, tokens=None) == E
    assert _score(L, target=36) == E                      # misaligned logits
    assert _score(L, uniforms=None) == E                  # rejection mode needs uniforms
    assert b"uniforms" in L.ppow_last_error()
    P = binding.PpowParams
    assert _score(L, params=P(0.0, 0.5, 1.0, 0, 0, 0, 0.0)) == E
    assert _score(L, params=P(float("nan"), 0.5, 1.0, 0, 0, 0, 0.0)) == E
    assert _score(L, params=P(0.05, 0.5, 1.0, 2, 0, 0, 0.0)) == E      # verify enum
    assert _score(L, params=P(0.05, 0.5, 1.0, 0, 8, 0, 0.0)) == E      # unknown flag
    assert _score(L, params=P(0.05, 0.5, 1.0, 0, 1, 0, 0.0)) == E      # flag w/o output
    O = binding.PpowOutputs
    assert _score(L, outs=O(*([4096] * 3 + [None] * 15))) == E           # a required output missing
    assert _score(L, outs=O(*([4096] * 4 + [None] * 4 + [4096] + [None] * 9))) == E   # output w/o flag
    assert _score(L, outs=O(*([4096] * 4 + [None] * 7 + [4096] + [None] * 6))) == E   # reverse_kl w/o flag
    assert _score(L, outs=O(*([4096] * 4 + [None] * 12 + [4096, None]))) == E        # group output w/o group
    adv = O(*([4096] * 4 + [None] * 11 + [4096] + [None] * 2))
    assert _score(L, outs=adv) == E                                      # advantage w/o group size
    assert _score(L, outs=adv, params=P(0.05, 0.5, 1.0, 0, 0, 3, 1e-6)) == E   # 3 does not divide B=4
    assert _score(L, outs=adv, params=P(0.05, 0.5, 1.0, 0, 0, 2, -1.0)) == E
    W = binding.PPOW_ERR_WORKSPACE
    assert _score(L, ws=None) == W
    assert _score(L, ws=4100) == W
    assert _score(L, ws_bytes=8) == W
    assert b"workspace" in L.ppow_last_error()


def test_sequence_argument_errors_return_before_any_launch():
    L = ppow.lib()
    E, W = binding.PPOW_ERR_INVALID_ARG, binding.PPOW_ERR_WORKSPACE

    def seq(draft=16, target=32, N=2, T=8, V=100, dtype=0, K=4, u=None, rho=1.0, mix=None, crit=None,
            score=4096, start=None, ws=4096, ws_bytes=1 << 24):
        return L.ppow_adaw_sequence(draft, target, N, T, V, dtype, K, u, rho, mix, crit, score, start,
                                    ws, ws_bytes, None)
    assert L.ppow_adaw_sequence_workspace_bytes(64, 2048, 128256, 1) == (1 << 20) + 64 * 2048 * 32
    assert L.ppow_adaw_sequence_workspace_bytes(2, 0, 100, 0) == 0
    assert seq(K=0) == E and seq(K=9) == E and seq(T=0) == E and seq(V=1) == E and seq(dtype=3) == E
    assert seq(N=-1) == E and seq(draft=None) == E and seq(score=None) == E and seq(target=40) == E
    assert seq(start=4096) == E                      # sampling needs uniforms
    assert seq(start=4096, u=8192, rho=0.4) == E     # a curriculum fraction below 1 needs its draws
    assert seq(start=4096, u=8192, rho=1.5, mix=64) == E and seq(start=4096, u=8192, rho=-0.1, mix=64) == E
    assert seq(start=4096, u=8192, rho=float("nan"), mix=64) == E
    assert seq(ws=None) == W and seq(ws_bytes=64) == W
    assert seq(N=0, draft=None, target=None, score=None) == binding.PPOW_OK


def test_select_argument_errors_return_before_any_launch():
    L = ppow.lib()
    E, W = binding.PPOW_ERR_INVALID_ARG, binding.PPOW_ERR_WORKSPACE
    assert L.ppow_select_windows(16, 10, 0, 32, None, 4096, 1 << 20, None) == E
    assert L.ppow_select_windows(16, 10, 11, 32, None, 4096, 1 << 20, None) == E
    assert L.ppow_select_windows(16, 0, 1, 32, None, 4096, 1 << 20, None) == E
    assert L.ppow_select_windows(None, 10, 5, 32, None, 4096, 1 << 20, None) == E
    assert L.ppow_select_windows(16, 10, 5, None, None, 4096, 1 << 20, None) == E
    assert L.ppow_select_windows(16, 10, 5, 32, None, None, 1 << 20, None) == W
    assert L.ppow_select_windows(16, 10, 5, 32, None, 4096, 8, None) == W


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(2, 2, 8)
    with pytest.raises(RuntimeError, match="no CPU path"):
        ppow.ppow_score_windows(x, x, torch.zeros(2, 2, dtype=torch.int32), torch.zeros(2, 2),
                                cost_ratio=0.1)
    with pytest.raises(RuntimeError, match="no CPU path"):
        ppow.ppow_select_windows(torch.zeros(8), 2)


def test_static_entry_point_rejects_on_the_host_what_it_can():
    """Bad arguments and sizes beyond the built-in scratch are refused before any device call."""
    L = ppow.lib()
    p = binding.PpowParams(0.05, 0.5, 1.0, 0, 0, 0, 0.0)
    o = binding.PpowOutputs(*([4096] * 4 + [None] * 14))

    def call(B=4, K=2, V=100, draft=16, params=p):
        return L.ppow_score_windows_static(draft, 32, 48, 64, None, B, K, V, 0,
                                           ctypes.byref(params), ctypes.byref(o), None)

    assert call(draft=None) == binding.PPOW_ERR_INVALID_ARG
    assert call(K=65) == binding.PPOW_ERR_INVALID_ARG
    assert call(params=binding.PpowParams(-1.0, 0.5, 1.0, 0, 0, 0, 0.0)) == binding.PPOW_ERR_INVALID_ARG
    assert call(B=binding.PPOW_STATIC_MAX_ROWS // 2 + 1, K=2) == binding.PPOW_ERR_UNSUPPORTED
    assert b"built-in scratch" in L.ppow_last_error()
    assert call(B=0) == binding.PPOW_OK
    assert L.ppow_release() == binding.PPOW_OK          # nothing held: a no-op
