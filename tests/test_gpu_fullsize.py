"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot score 10^10 logits in a test, so each full-size run is checked on
a seeded sample of windows the oracle scores one by one (from a device-to-host copy
of the same stored bytes), on properties that hold at any size, and with an exact
check of the top-M selection against a full sort of the GPU's own fp32 scores.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14978_amd as ppow
from workloads import WORKLOADS, generate, generate_sequences

from parity import check_selection, compare, run_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SAMPLE = 512


def _score_chunk(w, d, sbuf):
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if w.expected_accept else 0
    assert code == (ppow.PPOW_BF16 if d["target_logits"].dtype == torch.bfloat16 else ppow.PPOW_F32)
    ppow.ppow_score_windows(
        d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
        cost_ratio=w.cost_ratio, prox_eps=w.prox_eps, prox_eta=w.prox_eta,
        verify=ppow.PPOW_VERIFY_GREEDY if w.verify == "greedy" else ppow.PPOW_VERIFY_REJECTION,
        flags=flags, buffers=sbuf)


def _check_sample(w, d, out, w0, seed):
    """Oracle on SAMPLE seeded windows of this chunk; `out` holds all windows, chunk at w0."""
    rng = np.random.default_rng(seed)
    pick = np.sort(rng.choice(w.B, size=min(SAMPLE, w.B), replace=False))
    idx = torch.from_numpy(pick).to(DEV)
    sub = {k: (None if v is None else v.index_select(0, idx).contiguous()) for k, v in d.items()}
    ref = run_oracle(sub, cost_ratio=w.cost_ratio, verify=w.verify, prox_eps=w.prox_eps,
                     prox_eta=w.prox_eta, expected_accept=w.expected_accept)

    class Picked:
        pass
    got = Picked()
    sel = idx + w0
    for name in ("accepted_len", "r_speedup", "r_proximity", "adaw_score"):
        setattr(got, name, getattr(out, name).index_select(0, sel))
    for name in ("delta", "kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok",
                 "expected_accept"):
        t = getattr(out, name)
        setattr(got, name, None if t is None else t.index_select(0, sel))
    compare(got, ref, w.dtype, w.V, w.expected_accept)


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
def test_full_size_workload(name):
    w = WORKLOADS[name]
    total = w.B * w.chunks
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if w.expected_accept else 0
    optional = ("delta", "kl", "confidence", "accept_prob") + (("expected_accept",) if w.expected_accept else ())
    out = ppow.ScoreBuffers(total, w.K, w.V, code, DEV, optional, flags)
    for c in range(w.chunks):
        print(f"{name}: chunk {c + 1}/{w.chunks}", flush=True)
        d = generate(w, device=DEV, chunk=c)
        _score_chunk(w, d, out.window_slice(c * w.B, (c + 1) * w.B))
        torch.cuda.synchronize()
        _check_sample(w, d, out, c * w.B, seed=w.seed + c)
        del d
        torch.cuda.empty_cache()
    _check_properties(w, out)
    idx = check_selection(out.adaw_score, w.M)          # global top-M over every chunk
    assert len(set(idx.tolist())) == w.M


def test_full_size_sequence_mode():
    """Sequence-mode ADAW at the benchmark's size: two sampled sequences against the oracle,
    the sampler and the selection exactly on the GPU's own scores."""
    from parity import RTOL, assert_close
    w = WORKLOADS["sequence_bf16_128k"]
    N, T, K = w.B, w.seq_len, w.K
    d = generate_sequences(w, device=DEV)
    out = ppow.ppow_adaw_sequence(d["draft_logits"], d["target_logits"], K, d["uniforms"])
    torch.cuda.synchronize()
    for n in (3, N - 1):
        print(f"sequence {n}", flush=True)
        v_ref, s_ref = oracle.adaw_sequence(d["draft_logits"][n:n + 1].cpu(), d["target_logits"][n:n + 1].cpu(), K)
        assert_close("criticality", out.criticality[n].cpu(), v_ref, RTOL[w.dtype])
        assert_close("window_score", out.window_score[n].cpu(), s_ref, RTOL[w.dtype])
    s_gpu = out.window_score.cpu().numpy().astype(np.float64)
    picks = oracle.sample_starts(s_gpu, d["uniforms"].cpu().numpy().astype(np.float64))
    assert np.array_equal(out.sampled_start.cpu().numpy(), picks)
    assert s_gpu.min() >= 0 and np.all(np.isfinite(s_gpu))
    idx = check_selection(out.window_score.view(-1), w.M)
    assert len(set(idx.tolist())) == w.M
