"""The synthetic generator keeps the method's decisions unambiguous (CPU, small sizes).

The margins are checked with the oracle, which the generator never calls.
"""
import numpy as np
import pytest
import torch

import oracle
import importlib

from workloads import WORKLOADS, generate, generate_all
from workloads.generate import ACCEPT_MARGIN, ARGMAX_MARGIN, GAP_MARGIN, SCORE_GAP

generator = importlib.import_module("workloads.generate")

SMALL = [("tiny_f32", 32), ("greedy_bf16_32k", 24), ("rejection_bf16_128k", 6),
         ("twopass_f32_152k", 5), ("stream_bf16_128k", 4)]


@pytest.mark.parametrize("name,B", SMALL)
def test_margins_hold_and_shapes_match(name, B):
    w = WORKLOADS[name].scaled(B)
    d = generate(w)
    a, b = d["target_logits"], d["draft_logits"]
    assert a.shape == b.shape == (B, w.K, w.V)
    assert a.dtype == b.dtype == (torch.bfloat16 if w.dtype == "bf16" else torch.float32)
    assert d["draft_tokens"].dtype == torch.int32 and d["draft_tokens"].shape == (B, w.K)
    assert int(d["draft_tokens"].min()) >= 0 and int(d["draft_tokens"].max()) < w.V
    top2 = torch.topk(a.float(), 2, -1).values
    assert float((top2[..., 0] - top2[..., 1]).min()) >= ARGMAX_MARGIN
    greedy = w.verify == "greedy"
    u = None if greedy else d["uniforms"].numpy()
    r = oracle.score_windows(b, a, d["draft_tokens"].numpy(), u, cost_ratio=w.cost_ratio,
                             verify=oracle.GREEDY if greedy else oracle.REJECTION)
    if not greedy:
        assert d["uniforms"].dtype == torch.float32
        assert np.abs(u.astype(np.float64) - r.accept_prob).min() >= ACCEPT_MARGIN * (1 - 1e-6)
    assert np.abs(r.delta - w.prox_eps).min() >= GAP_MARGIN * (1 - 1e-6)
    assert np.all(np.isfinite(r.adaw_score)) and np.all(r.adaw_score >= 0)
    if w.chunks == 1 and w.M < B:
        assert _relative_gap(r.adaw_score, w.M) >= SCORE_GAP * (1 - 1e-6)


def _relative_gap(scores, M):
    top = np.sort(np.asarray(scores, dtype=np.float64))[::-1]
    return (top[M - 1] - top[M]) / abs(top[M - 1])


def _oracle_scores(w, d):
    greedy = w.verify == "greedy"
    r = oracle.score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"].numpy(),
                             None if greedy else d["uniforms"].numpy(), cost_ratio=w.cost_ratio,
                             verify=oracle.GREEDY if greedy else oracle.REJECTION)
    return r, r.adaw_score


@pytest.mark.parametrize("chunks,required", [(1, 0.08), (3, 0.03)])
def test_selection_gap_is_enforced_by_redrawing_windows(monkeypatch, chunks, required):
    """With the required gap raised far above what random scores give, the generator has to
    draw boundary windows again; the gap then holds on the oracle's scores, over all chunks,
    and the redrawn windows keep their own margins."""
    w = WORKLOADS["tiny_f32"].scaled(24, M=9, chunks=chunks)
    plain = [generate(w, chunk=c) for c in range(chunks)]
    before = np.concatenate([_oracle_scores(w, d)[1] for d in plain])
    assert _relative_gap(before, w.M) < required          # the case needs the enforcement
    monkeypatch.setattr(generator, "SCORE_GAP", required)
    fixed = [d for _, d in generate_all(w)]
    results = [_oracle_scores(w, d)[0] for d in fixed]
    after = np.concatenate([r.adaw_score for r in results])
    assert _relative_gap(after, w.M) >= required * (1 - 1e-6)
    # only windows of the last chunk were touched, and only a few of them
    for c in range(chunks - 1):
        assert torch.equal(plain[c]["target_logits"], fixed[c]["target_logits"])
    changed = (plain[-1]["target_logits"] != fixed[-1]["target_logits"]).flatten(1).any(-1)
    assert 1 <= int(changed.sum()) <= 12
    last = results[-1]
    u = fixed[-1]["uniforms"].numpy().astype(np.float64)
    assert np.abs(u - last.accept_prob).min() >= ACCEPT_MARGIN * (1 - 1e-6)
    assert np.abs(last.delta - w.prox_eps).min() >= GAP_MARGIN * (1 - 1e-6)


def test_generation_is_seeded_and_chunks_differ():
    w = WORKLOADS["stream_bf16_128k"].scaled(2)
    d0, d0b, d1 = generate(w, chunk=0), generate(w, chunk=0), generate(w, chunk=1)
    assert torch.equal(d0["target_logits"], d0b["target_logits"])
    assert torch.equal(d0["draft_tokens"], d0b["draft_tokens"])
    assert not torch.equal(d0["target_logits"], d1["target_logits"])
