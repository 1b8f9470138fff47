"""The synthetic generator keeps the method's decisions unambiguous (CPU, small sizes).

The margins are checked with the oracle, which the generator never calls.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import WORKLOADS, generate
from workloads.generate import ACCEPT_MARGIN, ARGMAX_MARGIN, GAP_MARGIN

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


def test_generation_is_seeded_and_chunks_differ():
    w = WORKLOADS["stream_bf16_128k"].scaled(2)
    d0, d0b, d1 = generate(w, chunk=0), generate(w, chunk=0), generate(w, chunk=1)
    assert torch.equal(d0["target_logits"], d0b["target_logits"])
    assert torch.equal(d0["draft_tokens"], d0b["draft_tokens"])
    assert not torch.equal(d0["target_logits"], d1["target_logits"])
