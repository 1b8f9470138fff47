"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every window of every workload is scored by the oracle too: the stored logits go to the
host in slices of SLICE windows (a few GB), so host memory never limits the size.  Accepted
lengths and proximity rewards are compared exactly, floats within the stated tolerance, on
all windows; the global top-M is compared with the selection the oracle makes on its own
double-precision scores (equal as sets: the generator keeps the M-th and the (M+1)-th score
1e-4 apart, far above the error of a score); each call runs twice and must repeat bit for
bit.  The largest observed deviation per output is printed.
"""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2605_14978_amd as ppow
from workloads import WORKLOADS, generate_all, generate_sequences
from workloads.generate import SCORE_GAP

from parity import ErrorReport, check_selection, compare, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SLICE = 1024
OUTPUTS = ("accepted_len", "r_speedup", "r_proximity", "adaw_score")
OPTIONAL = ("delta", "kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok")


def _score_chunk(w, d, sbuf):
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if w.expected_accept else 0
    assert code == (ppow.PPOW_BF16 if d["target_logits"].dtype == torch.bfloat16 else ppow.PPOW_F32)
    ppow.ppow_score_windows(
        d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
        cost_ratio=w.cost_ratio, prox_eps=w.prox_eps, prox_eta=w.prox_eta,
        verify=ppow.PPOW_VERIFY_GREEDY if w.verify == "greedy" else ppow.PPOW_VERIFY_REJECTION,
        flags=flags, buffers=sbuf)
    torch.cuda.synchronize()
    assert sbuf.status() == 0, "the cluster kernel reported an expired wait"


def _check_properties(w, out):
    k = out.accepted_len.cpu().numpy()
    assert k.min() >= 0 and k.max() <= w.K
    kf = k.astype(np.float32)
    expect = kf / (kf * np.float32(w.cost_ratio) + np.float32(1.0))
    np.testing.assert_allclose(out.r_speedup.cpu().numpy(), expect, rtol=3e-7)
    rp = out.r_proximity.cpu().numpy()
    assert np.all((rp == 0) | (rp == np.float32(w.prox_eta)))
    assert np.all(rp[k > 0] == 0)                       # the proximity reward is gated on k = 0
    s = out.adaw_score.cpu().numpy()
    assert np.all(np.isfinite(s)) and s.min() >= 0
    assert 0 < k.mean() < w.K                           # truncation happens, but not always


@pytest.mark.parametrize("name", ["greedy_bf16_32k", "rejection_bf16_128k", "twopass_f32_152k",
                                  "stream_bf16_128k"])
def test_full_size_workload(name, capsys):
    w = WORKLOADS[name]
    total = w.B * w.chunks
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if w.expected_accept else 0
    optional = OPTIONAL + (("expected_accept",) if w.expected_accept else ())
    out = ppow.ScoreBuffers(total, w.K, w.V, code, DEV, optional, flags)
    again = ppow.ScoreBuffers(w.B, w.K, w.V, code, DEV, optional, flags)
    oracle_scores = np.empty(total, dtype=np.float64)
    report = ErrorReport()
    t_start = time.perf_counter()

    def say(text):                       # progress past pytest's capture: a long test is not a hung one
        with capsys.disabled():
            print(f"\n[{name} {time.perf_counter() - t_start:5.0f} s] {text}", end="", flush=True)

    for c, d in generate_all(w, device=DEV):
        w0 = c * w.B
        mine = out.window_slice(w0, w0 + w.B)
        _score_chunk(w, d, mine)
        _score_chunk(w, d, again)                        # same launch again: bit for bit
        for field in OUTPUTS + optional:
            assert torch.equal(getattr(mine, field), getattr(again, field)), f"{field} does not repeat"
        for s0 in range(0, w.B, SLICE):
            s1 = min(w.B, s0 + SLICE)
            sub = {k: (None if v is None else v[s0:s1]) for k, v in d.items()}
            ref = run_oracle(sub, cost_ratio=w.cost_ratio, verify=w.verify, prox_eps=w.prox_eps,
                             prox_eta=w.prox_eta, expected_accept=w.expected_accept)
            compare(out.window_slice(w0 + s0, w0 + s1), ref, w.dtype, w.V, w.expected_accept,
                    report=report)
            oracle_scores[w0 + s0:w0 + s1] = ref.adaw_score
            say(f"chunk {c + 1}/{w.chunks}: windows {w0 + s0}..{w0 + s1} of {total} match the oracle")
        del d, sub
        torch.cuda.empty_cache()
    _check_properties(w, out)
    top = np.sort(oracle_scores)[::-1]
    gap = (top[w.M - 1] - top[w.M]) / top[w.M - 1]
    say(f"relative tolerance each output would have needed at its absolute floor: {report}")
    say(f"top-{w.M} boundary: oracle scores {top[w.M - 1]:.9g} / {top[w.M]:.9g}, relative gap {gap:.2e}\n")
    assert gap >= SCORE_GAP * (1 - 1e-6)
    idx = check_selection(out.adaw_score, w.M, oracle_scores, 1e-4, exact_sets=True)
    assert len(set(idx.tolist())) == w.M


def test_full_size_sequence_mode(capsys):
    """Sequence-mode ADAW at the benchmark's size: every sequence against the oracle (eight
    at a time), the sampler exactly on the GPU's own scores, the selection against the
    oracle's scores within the tolerance band (sequence inputs carry no selection gap)."""
    from parity import ATOL_DIVERGENCE, RTOL, assert_close
    w = WORKLOADS["sequence_bf16_128k"]
    N, T, K = w.B, w.seq_len, w.K
    d = generate_sequences(w, device=DEV)
    out = ppow.ppow_adaw_sequence(d["draft_logits"], d["target_logits"], K, d["uniforms"])
    again = ppow.ppow_adaw_sequence(d["draft_logits"], d["target_logits"], K, d["uniforms"])
    torch.cuda.synchronize()
    for field in ("criticality", "window_score", "sampled_start"):
        assert torch.equal(getattr(out, field), getattr(again, field)), f"{field} does not repeat"
    report = ErrorReport()
    s_ref_all = np.empty((N, T - K + 1), dtype=np.float64)
    for n0 in range(0, N, 8):
        n1 = min(N, n0 + 8)
        v_ref, s_ref = oracle.adaw_sequence(d["draft_logits"][n0:n1].cpu(), d["target_logits"][n0:n1].cpu(), K)
        assert_close("criticality", out.criticality[n0:n1].cpu(), v_ref, RTOL[w.dtype], ATOL_DIVERGENCE)
        assert_close("window_score", out.window_score[n0:n1].cpu(), s_ref, RTOL[w.dtype], ATOL_DIVERGENCE)
        report.add("criticality", out.criticality[n0:n1].cpu(), v_ref, ATOL_DIVERGENCE)
        report.add("window_score", out.window_score[n0:n1].cpu(), s_ref, ATOL_DIVERGENCE)
        s_ref_all[n0:n1] = s_ref
        with capsys.disabled():
            print(f"\n[sequence_bf16_128k] sequences {n0}..{n1} of {N} match the oracle", end="", flush=True)
    with capsys.disabled():
        print(f"\n[sequence_bf16_128k] relative tolerance needed at the absolute floor: {report}", flush=True)
    s_gpu = out.window_score.cpu().numpy().astype(np.float64)
    picks = oracle.sample_starts(s_gpu, d["uniforms"].cpu().numpy().astype(np.float64))
    assert np.array_equal(out.sampled_start.cpu().numpy(), picks)
    assert s_gpu.min() >= 0 and np.all(np.isfinite(s_gpu))
    idx = check_selection(out.window_score.view(-1), w.M, s_ref_all.reshape(-1), 1e-4)
    assert len(set(idx.tolist())) == w.M
