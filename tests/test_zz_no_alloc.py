"""ppow_score_windows_static -- the scoring entry point that allocates nothing -- against
ppow_score_windows, through the C ABI, on two calls in a row (the second with a smaller
input, so that what the first call left in the built-in scratch must not show)."""
import pytest
import torch

import paper_2605_14978_amd as ppow
from paper_2605_14978_amd import binding
from workloads import WORKLOADS, generate

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

PER_POSITION = ("kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok")


def _both_entry_points(w, d, second_pass):
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if second_pass else 0
    optional = ("delta",) + PER_POSITION + (("expected_accept",) if second_pass else ())
    verify = ppow.PPOW_VERIFY_GREEDY if w.verify == "greedy" else ppow.PPOW_VERIFY_REJECTION
    args = (d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"])
    kw = dict(cost_ratio=w.cost_ratio, prox_eps=w.prox_eps, prox_eta=w.prox_eta, verify=verify,
              flags=flags)
    ref = ppow.ppow_score_windows(*args, optional=optional, **kw)
    kernel_ref = ppow.last_row_kernel()
    torch.cuda.synchronize()
    out = ppow.ScoreBuffers(w.B, w.K, w.V, code, DEV, optional, flags, workspace=False)
    before = torch.cuda.memory_allocated()
    ppow.ppow_score_windows_static(*args, buffers=out, **kw)
    assert torch.cuda.memory_allocated() == before
    assert ppow.last_row_kernel() == kernel_ref
    torch.cuda.synchronize()
    assert ref.status() == 0 and out.status() == 0
    # Same kernels on the same inputs in a fixed summation order: the bar for floats is the
    # oracle tolerance, what is observed is bitwise equality.
    for name in ("accepted_len", "r_speedup", "r_proximity", "adaw_score") + optional:
        assert torch.equal(getattr(out, name), getattr(ref, name)), name
    return out


@pytest.mark.parametrize("name,second_pass", [("rejection_bf16_128k", False),
                                              ("twopass_f32_152k", True),
                                              ("greedy_bf16_32k", False)])
def test_static_scratch_entry_point_matches_the_workspace_one(name, second_pass):
    big = WORKLOADS[name].scaled(48)
    small = WORKLOADS[name].scaled(5)
    first = _both_entry_points(big, generate(big, device=DEV), second_pass)
    assert 0 < first.accepted_len.float().mean() < big.K
    _both_entry_points(small, generate(small, device=DEV), second_pass)


def test_static_scratch_limit_and_argument_errors():
    L = ppow.lib()
    w = WORKLOADS["tiny_f32"]
    d = generate(w, device=DEV)
    out = ppow.ScoreBuffers(w.B, w.K, w.V, ppow.PPOW_F32, DEV, workspace=False)
    # one row too many for the built-in scratch: refused before anything is looked at
    K = 64
    B = ppow.PPOW_STATIC_MAX_ROWS // K + 1
    params = binding.PpowParams(0.05, 0.5, 1.0, 0, 0, 0, 0.0)
    outs = out.as_struct()
    import ctypes
    status = L.ppow_score_windows_static(
        d["draft_logits"].data_ptr(), d["target_logits"].data_ptr(), d["draft_tokens"].data_ptr(),
        d["uniforms"].data_ptr(), None, B, K, 1000, ppow.PPOW_F32, ctypes.byref(params),
        ctypes.byref(outs), None)
    assert status == binding.PPOW_ERR_UNSUPPORTED
    assert b"exceed" in L.ppow_last_error()
    status = L.ppow_score_windows_static(
        None, d["target_logits"].data_ptr(), d["draft_tokens"].data_ptr(),
        d["uniforms"].data_ptr(), None, w.B, w.K, w.V, ppow.PPOW_F32, ctypes.byref(params),
        ctypes.byref(outs), None)
    assert status == binding.PPOW_ERR_INVALID_ARG
    # exactly at the limit the call is accepted (B = 0 windows of it are launched: no-op sizes
    # are checked the same way)
    assert L.ppow_score_windows_static(None, None, None, None, None, 0, 4, 1000, ppow.PPOW_F32,
                                       ctypes.byref(params), ctypes.byref(outs), None) == 0
