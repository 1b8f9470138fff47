"""Seeded synthetic inputs for the window-scoring path.

Both the HIP library and the CPU oracle consume the tensors produced here (the
oracle from a device-to-host copy of the very same stored bytes).  This module
draws random logits, drafted tokens and uniforms with torch library routines and
keeps the decisions of the method unambiguous by construction:

  * target argmax margin: top-1 minus top-2 logit >= ARGMAX_MARGIN after
    rounding to the storage dtype (so greedy verification never hinges on a tie);
  * acceptance margin: |u - alpha| >= ACCEPT_MARGIN for every position, alpha
    being min(1, P(tok)/Q(tok)) evaluated with torch's float64 log_softmax;
  * proximity margin: |gap - eps| >= GAP_MARGIN for every window, the gap being
    the sum over positions of (max target logit - target logit of the drafted
    token) in float64;
  * selection margin: the M-th and the (M+1)-th largest window score of a workload
    differ by at least SCORE_GAP relative, the scores being evaluated with torch's
    float64 log_softmax.

The margin checks use torch float64 library calls only; their values are never
handed to either implementation.  The windows stand in for the logits that the
paper's draft/target pairs would produce on its evaluation suites, which are
not reproduced here.
"""
import math

import torch

from .configs import Workload

ARGMAX_MARGIN = 0.05
ACCEPT_MARGIN = 1e-3
GAP_MARGIN = 1e-3
SCORE_GAP = 1e-4           # relative gap between the M-th and the (M+1)-th largest window score
ROWS_PER_CHUNK = 1024      # generation granularity (rows of V logits)


def torch_dtype(w: Workload):
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def _zipf_prior(V, gen, device):
    """Additive unigram prior -1.1 * ln(1 + rank), rank a seeded permutation."""
    rank = torch.randperm(V, generator=gen, device=device).to(torch.float32)
    return -1.1 * torch.log1p(rank)


def _target_rows(w, n, gen, device, prior):
    if w.family == "boosted":
        a = torch.randn(n, w.V, generator=gen, device=device) * 3.0
        hot = torch.randint(0, w.V, (n,), generator=gen, device=device)
        a[torch.arange(n, device=device), hot] += 6.0
        return a
    a = torch.randn(n, w.V, generator=gen, device=device) * 2.5
    return a + prior


def _draft_rows(w, a, gen, device):
    n = a.shape[0]
    if w.family == "boosted":
        sigma = torch.rand(n, 1, generator=gen, device=device) * 1.8 + 0.2
        return a + torch.randn(n, w.V, generator=gen, device=device) * sigma
    if w.family == "tempered":
        temp = torch.rand(n, 1, generator=gen, device=device) * 0.8 + 0.7
        return a / temp + torch.randn(n, w.V, generator=gen, device=device) * 0.5
    # "zipf": log-normal noise scale per position, 10 % hard positions at sigma = 4
    sigma = torch.exp(torch.randn(n, 1, generator=gen, device=device) * 0.7 - 1.0)
    hard = torch.rand(n, 1, generator=gen, device=device) < 0.10
    sigma = torch.where(hard, torch.full_like(sigma, 4.0), sigma)
    return a + torch.randn(n, w.V, generator=gen, device=device) * sigma


def _enforce_argmax_margin(a_stored):
    """Raise the top-1 logit of rows whose stored top-2 gap is below the margin."""
    for it in range(8):
        top = torch.topk(a_stored.float(), 2, dim=-1)
        gap = top.values[:, 0] - top.values[:, 1]
        bad = torch.nonzero(gap < ARGMAX_MARGIN).flatten()
        if bad.numel() == 0:
            return
        bump = top.values[bad, 1] + 0.07 + 0.07 * it
        a_stored[bad, top.indices[bad, 0]] = bump.to(a_stored.dtype)
    raise RuntimeError("could not enforce the argmax margin")


def _sample_tokens(b_stored, gen, greedy_draft):
    if greedy_draft:
        return b_stored.float().argmax(-1)
    u = torch.rand(b_stored.shape, generator=gen, device=b_stored.device)
    gumbel = -torch.log(-torch.log(u.clamp_min(1e-30)).clamp_min(1e-30))
    return (b_stored.float() + gumbel).argmax(-1)       # Gumbel-max = categorical sample


def _make_windows(w, n_windows, gen, device, prior, dt, greedy):
    """Draw `n_windows` whole windows with the per-window margins enforced.

    Returns (target rows, draft rows, tokens, uniforms, window scores): the first two
    [n_windows*K, V] in the storage dtype, the last a float64 [n_windows] tensor of
    (1/K) sum_t C(P_t) KL(P_t||Q_t) from torch's float64 log_softmax, used only to keep the
    top-M boundary clear (enforce_selection_gap) and never handed to either implementation.
    """
    K = w.K
    n = n_windows * K
    a = _target_rows(w, n, gen, device, prior)
    b = _draft_rows(w, a, gen, device)
    a_st = a.to(dt)
    b_st = b.to(dt)
    del a, b
    _enforce_argmax_margin(a_st)
    a64 = a_st.double()
    amax = a64.max(-1).values
    logp = torch.log_softmax(a64, -1)
    logq = torch.log_softmax(b_st.double(), -1)
    del a64

    tok = _sample_tokens(b_st, gen, greedy_draft=greedy)
    for attempt in range(64):
        gap_t = amax - a_st.gather(1, tok[:, None])[:, 0].double()
        gap = gap_t.view(-1, K).sum(-1)
        bad_w = torch.nonzero((gap - w.prox_eps).abs() < GAP_MARGIN).flatten()
        if bad_w.numel() == 0:
            break
        bad_r = (bad_w[:, None] * K + torch.arange(K, device=device)[None, :]).flatten()
        tok[bad_r] = _sample_tokens(b_st[bad_r], gen, greedy_draft=False)
    else:
        raise RuntimeError("could not enforce the proximity margin")

    lp = logp.gather(1, tok[:, None])[:, 0]
    lq = logq.gather(1, tok[:, None])[:, 0]
    alpha = torch.exp(torch.clamp(lp - lq, max=0.0))
    p = torch.exp(logp)
    entropy = -(p * logp).sum(-1)
    logq -= logp                                     # in place: log Q - log P
    divergence = -(p * logq).sum(-1)
    del logp, logq, p
    score = ((1.0 - entropy / math.log(w.V)) * divergence).view(-1, K).mean(-1)
    u = torch.rand(n, generator=gen, device=device)
    for attempt in range(64):
        bad = torch.nonzero((u.double() - alpha).abs() < ACCEPT_MARGIN).flatten()
        if bad.numel() == 0:
            break
        u[bad] = torch.rand(bad.numel(), generator=gen, device=device)
    else:
        raise RuntimeError("could not enforce the acceptance margin")
    return a_st, b_st, tok, u, score


def _boundary(scores, M):
    """(rank order, relative gap between the M-th and the (M+1)-th largest score)."""
    order = torch.sort(scores, descending=True, stable=True).indices
    hi, lo = scores[order[M - 1]], scores[order[M]]
    return order, float((hi - lo) / hi.abs().clamp_min(1e-300))


def _generate(w: Workload, device, chunk, earlier_scores):
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed + chunk)
    dt = torch_dtype(w)
    B, K, V = w.B, w.K, w.V
    rows = B * K
    a_all = torch.empty(rows, V, dtype=dt, device=device)
    b_all = torch.empty(rows, V, dtype=dt, device=device)
    tok_all = torch.empty(rows, dtype=torch.int64, device=device)
    u_all = torch.empty(rows, dtype=torch.float32, device=device)
    score_all = torch.empty(B, dtype=torch.float64, device=device)
    prior = _zipf_prior(V, gen, device) if w.family != "boosted" else None
    greedy = w.verify == "greedy"

    windows_per_chunk = max(1, ROWS_PER_CHUNK // K)
    for w0 in range(0, B, windows_per_chunk):
        w1 = min(B, w0 + windows_per_chunk)
        r0, r1 = w0 * K, w1 * K
        a_all[r0:r1], b_all[r0:r1], tok_all[r0:r1], u_all[r0:r1], score_all[w0:w1] = \
            _make_windows(w, w1 - w0, gen, device, prior, dt, greedy)

    # Top-M boundary: the M-th and the (M+1)-th largest score over all windows of the workload
    # differ by at least SCORE_GAP (relative), so that the selected set cannot hinge on float
    # rounding.  Decided when the last chunk is drawn, with the float64 scores of the earlier
    # chunks at hand: the window of this chunk nearest in rank to the boundary is drawn again
    # (fresh sub-seed) until the gap holds.
    total = B * w.chunks
    if chunk == w.chunks - 1 and w.M < total and (w.chunks == 1 or earlier_scores is not None):
        offset = total - B
        for attempt in range(64):
            scores = score_all if w.chunks == 1 else torch.cat([earlier_scores.to(device), score_all])
            order, gap = _boundary(scores, w.M)
            if gap >= SCORE_GAP:
                break
            rank = torch.empty_like(order)
            rank[order] = torch.arange(total, device=device)
            # distance in rank from the boundary between positions M-1 and M; the (M+1)-th
            # window itself (rank M) wins a tie with the M-th
            dist = (rank[offset:].double() - (w.M - 0.25)).abs()
            victim = int(dist.argmin())
            sub = torch.Generator(device=device)
            sub.manual_seed((w.seed + chunk) * 1_000_003 + 7919 * (attempt + 1) + victim)
            r0 = victim * K
            a_all[r0:r0 + K], b_all[r0:r0 + K], tok_all[r0:r0 + K], u_all[r0:r0 + K], \
                score_all[victim:victim + 1] = _make_windows(w, 1, sub, device, prior, dt, greedy)
        else:
            raise RuntimeError("could not enforce the selection gap")

    return {
        "target_logits": a_all.view(B, K, V),
        "draft_logits": b_all.view(B, K, V),
        "draft_tokens": tok_all.to(torch.int32).view(B, K),
        "uniforms": None if greedy else u_all.view(B, K),
    }, score_all


def generate(w: Workload, device="cpu", chunk: int = 0):
    """Inputs of one scoring call (chunk `chunk` of the workload).

    Returns a dict of tensors on `device`:
      target_logits, draft_logits  [B, K, V]  in the workload's storage dtype
      draft_tokens                 [B, K]     int32
      uniforms                     [B, K]     float32 (None for greedy verification)
    A workload of one chunk carries the top-M score gap; one of several chunks carries it only
    when its chunks are drawn in order by generate_all (the gap is a property of all of them).
    """
    return _generate(w, device, chunk, None)[0]


def generate_all(w: Workload, device="cpu"):
    """Yield (chunk index, inputs) for every chunk of the workload, in order, with the top-M
    score gap enforced over all of them (the last chunk may differ in one or a few windows from
    what generate(w, chunk=last) returns)."""
    seen = []
    for c in range(w.chunks):
        earlier = torch.cat(seen) if seen else torch.empty(0, dtype=torch.float64)
        d, scores = _generate(w, device, c, earlier if w.chunks > 1 else None)
        seen.append(scores.cpu())
        yield c, d


def generate_sequences(w: Workload, device="cpu"):
    """Inputs of sequence-mode ADAW: [N, T, V] teacher-forced logits and one uniform per sequence."""
    from dataclasses import replace
    as_windows = replace(w, K=w.seq_len, seq_len=0)           # one "window" per sequence
    d = generate(as_windows, device=device)
    gen = torch.Generator(device=torch.device(device))
    gen.manual_seed(w.seed + 7919)
    return {"target_logits": d["target_logits"], "draft_logits": d["draft_logits"],
            "uniforms": torch.rand(w.B, generator=gen, device=device)}


def accepted_length_histogram(accepted_len, K):
    """Counts of windows by accepted length 0..K (a report, not a check)."""
    return torch.bincount(accepted_len.to(torch.int64).cpu(), minlength=K + 1).tolist()


def logit_gigabytes(w: Workload) -> float:
    return w.B * w.logit_bytes_per_window / 1e9


def describe(w: Workload) -> str:
    return (f"{w.name}: {w.dtype} B={w.B}x{w.chunks} K={w.K} V={w.V} {w.verify} "
            f"gamma={w.cost_ratio} M={w.M} seed={w.seed} "
            f"({logit_gigabytes(w) * w.chunks:.2f} GB of logits, "
            f"{math.ceil(w.logit_bytes_per_window / 1024)} KiB per window)")
