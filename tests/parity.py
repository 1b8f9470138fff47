"""Shared helpers of the GPU parity tests: run libppow and the oracle on the same
stored inputs and compare element by element.

Tolerances: |gpu - oracle| <= rtol*|oracle| + atol.
  rtol 1e-4 for fp32 AND for bf16 logits.  (The task allows 2e-3 for bf16; both sides read
  the same stored bits and the kernel's arithmetic is fp32 either way, so bf16 inputs are held
  to the fp32 bound.)
  atol 1e-6 (times ln V for sums of log-probabilities), except for the divergences and what
  is built from them (kl, reverse_kl, criticality, window scores): 4e-6.  A divergence is what
  is left after two log-sum-exps of size ~10 cancel; each comes from an fp32 sum over the
  vocabulary whose relative error is a few 2^-24 * sqrt(additions per lane) ~ 5e-7 when one
  lane holds most of the probability, plus 2^-23 per v_exp_f32 and 2^-22 from the rounding
  of the exponents: ~1e-6 per side, 2e-6 for the difference, doubled for margin.  Observed
  worst case over the 1.4 million rows of the full-size workloads: 1.3e-6.
Integer results (accepted length, argmax-driven decisions, selected indices) are
compared exactly.
"""
import math

import numpy as np
import torch

import oracle
import paper_2605_14978_amd as ppow

RTOL = {"f32": 1e-4, "bf16": 1e-4}
ATOL = 1e-6
ATOL_DIVERGENCE = 4e-6

PER_POSITION = ("kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok")
POLICY_TERMS = ("reverse_kl", "alignment")


def dtype_name(t):
    return "bf16" if t.dtype == torch.bfloat16 else "f32"


def run_gpu(d, *, cost_ratio, verify, prox_eps=0.5, prox_eta=1.0, expected_accept=False,
            ref_logprob=None, optional=None, policy_terms=False, rollout_group=0, adv_delta=1e-6):
    opt = list(optional if optional is not None else ("delta",) + PER_POSITION)
    flags = 0
    if expected_accept:
        flags |= ppow.PPOW_FLAG_EXPECTED_ACCEPT
        opt.append("expected_accept")
    if policy_terms:
        flags |= ppow.PPOW_FLAG_POLICY_TERMS
        opt += list(POLICY_TERMS) + ["reverse_kl_mean", "alignment_mean"]
    if rollout_group:
        opt += ["advantage", "group_best_len", "group_best_index"]
    out = ppow.ppow_score_windows(
        d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"], ref_logprob,
        cost_ratio=cost_ratio, prox_eps=prox_eps, prox_eta=prox_eta,
        verify=ppow.PPOW_VERIFY_GREEDY if verify == "greedy" else ppow.PPOW_VERIFY_REJECTION,
        flags=flags, rollout_group=rollout_group, adv_delta=adv_delta, optional=tuple(opt))
    torch.cuda.synchronize()
    assert out.status() == 0, "the cluster kernel reported an expired wait"
    return out


def run_oracle(d, *, cost_ratio, verify, prox_eps=0.5, prox_eta=1.0, expected_accept=False,
               ref_logprob=None, policy_terms=False, **_unused):
    want = list(PER_POSITION)
    if expected_accept:
        want.append("expected_accept")
    if policy_terms:
        want += list(POLICY_TERMS)
    u = d["uniforms"]
    return oracle.score_windows(
        d["draft_logits"].cpu(), d["target_logits"].cpu(), d["draft_tokens"].cpu().numpy(),
        None if u is None else u.cpu().numpy(),
        None if ref_logprob is None else ref_logprob.cpu().numpy(),
        cost_ratio=cost_ratio, prox_eps=prox_eps, prox_eta=prox_eta,
        verify=oracle.GREEDY if verify == "greedy" else oracle.REJECTION, want=tuple(want))


def _atol_of(name, V):
    if name.startswith("logp"):
        return ATOL * math.log(V)
    return ATOL_DIVERGENCE if name == "kl" else ATOL


def assert_close(name, got, ref, rtol, atol=ATOL):
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + atol
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (
        f"{name}: element {worst} got {got[worst]!r} ref {ref[worst]!r} "
        f"err {err[worst]:.3e} > bound {bound[worst]:.3e}")


class ErrorReport:
    """Largest observed deviation per output, accumulated over calls: for every element the
    relative tolerance that |got - ref| <= rtol*|ref| + atol would have needed."""

    def __init__(self):
        self.needed = {}

    def add(self, name, got, ref, atol=ATOL):
        got = np.asarray(got, dtype=np.float64).reshape(-1)
        ref = np.asarray(ref, dtype=np.float64).reshape(-1)
        excess = np.maximum(np.abs(got - ref) - atol, 0.0)
        with np.errstate(divide="ignore", invalid="ignore"):
            need = np.where(excess > 0, excess / np.abs(ref), 0.0)
        worst = float(need.max()) if need.size else 0.0
        self.needed[name] = max(self.needed.get(name, 0.0), worst)

    def __str__(self):
        return ", ".join(f"{k} {v:.1e}" for k, v in self.needed.items())


def compare(gpu, ref, dname, V, expected_accept=False, report=None, rtol=None):
    """Element-by-element comparison of one scoring call against the oracle."""
    rtol = RTOL[dname] if rtol is None else rtol
    if report is not None:
        report.add("r_speedup", gpu.r_speedup.cpu(), ref.r_speedup)
        report.add("adaw_score", gpu.adaw_score.cpu(), ref.adaw_score, ATOL_DIVERGENCE)
        if gpu.delta is not None:
            report.add("delta", gpu.delta.cpu(), ref.delta, ATOL * math.log(V))
        for name in PER_POSITION:
            if getattr(gpu, name) is not None:
                report.add(name, getattr(gpu, name).cpu(), getattr(ref, name), _atol_of(name, V))
        if expected_accept:
            report.add("expected_accept", gpu.expected_accept.cpu(), ref.expected_accept)
    assert np.array_equal(gpu.accepted_len.cpu().numpy(), ref.accepted_len), "accepted_len differs"
    assert_close("r_speedup", gpu.r_speedup.cpu(), ref.r_speedup, rtol)
    assert np.array_equal(gpu.r_proximity.cpu().numpy().astype(np.float64), ref.r_proximity), \
        "r_proximity differs"
    assert_close("adaw_score", gpu.adaw_score.cpu(), ref.adaw_score, rtol, ATOL_DIVERGENCE)
    if gpu.delta is not None:
        assert_close("delta", gpu.delta.cpu(), ref.delta, rtol, ATOL * math.log(V))
    for name in PER_POSITION:
        t = getattr(gpu, name)
        if t is not None:
            assert_close(name, t.cpu(), getattr(ref, name), rtol, _atol_of(name, V))
    if expected_accept:
        assert_close("expected_accept", gpu.expected_accept.cpu(), ref.expected_accept, rtol)
    if getattr(gpu, "reverse_kl", None) is not None:
        assert_close("reverse_kl", gpu.reverse_kl.cpu(), ref.reverse_kl, rtol, ATOL_DIVERGENCE)
        assert_close("alignment", gpu.alignment.cpu(), ref.alignment, rtol)
        assert_close("reverse_kl_mean", gpu.reverse_kl_mean.cpu(), ref.reverse_kl.mean(-1), rtol,
                     ATOL_DIVERGENCE)
        assert_close("alignment_mean", gpu.alignment_mean.cpu(), ref.alignment.mean(-1), rtol)


def compare_group_best(gpu, ref, group):
    """Best candidate per group: exact."""
    best, idx = oracle.group_best(ref.accepted_len, group)
    assert np.array_equal(gpu.group_best_len.cpu().numpy(), best)
    assert np.array_equal(gpu.group_best_index.cpu().numpy(), idx)


def compare_advantage(gpu, ref, group, adv_delta, rtol):
    """Group-relative advantages against the oracle's, group by group (Section 4.1)."""
    rewards = ref.r_speedup + ref.r_proximity
    expect = np.concatenate([oracle.group_advantage(rewards[i:i + group], adv_delta)
                             for i in range(0, rewards.size, group)])
    # The advantage divides by std + delta: the fp32 rounding of the two rewards (~6e-8
    # relative each) is amplified by |R| / (std + delta), so the floor is set by that, not by
    # the 1e-6 of the other outputs.
    std = np.repeat([rewards[i:i + group].std() for i in range(0, rewards.size, group)], group)
    floor = 4 * 6e-8 * np.abs(rewards).max() / (std + adv_delta)
    got = np.asarray(gpu.advantage.cpu(), dtype=np.float64)
    err = np.abs(got - expect)
    bound = rtol * np.abs(expect) + floor + ATOL
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (
        f"advantage: element {worst} got {got[worst]!r} ref {expect[worst]!r} "
        f"err {err[worst]:.3e} > bound {bound[worst]:.3e}")


def check_selection(gpu_scores, M, oracle_scores=None, rtol=None, exact_sets=False):
    """Selector exactness on the GPU's own fp32 scores, and (optionally) end-to-end
    agreement with the oracle's scores as sets, up to windows whose oracle score lies
    within the float tolerance of the M-th / (M+1)-th boundary.  With exact_sets the selected
    set must equal the oracle's outright (for inputs whose generator guarantees a boundary gap
    far above the error of the scores)."""
    sel = ppow.ppow_select_windows(gpu_scores, M)
    torch.cuda.synchronize()
    idx = sel.indices.cpu().numpy().astype(np.int64)
    s32 = gpu_scores.cpu().numpy()
    expect = oracle.select_windows(s32.astype(np.float64), M)
    assert np.array_equal(idx, expect), "selected indices differ from a full stable sort"
    assert np.array_equal(sel.scores.cpu().numpy(), s32[expect]), "selected scores differ"
    if oracle_scores is not None:
        ref_idx = oracle.select_windows(oracle_scores, M)
        B = oracle_scores.size
        if M < B:
            order = np.lexsort((np.arange(B), -oracle_scores))
            boundary = 0.5 * (oracle_scores[order[M - 1]] + oracle_scores[order[M]])
            tol = rtol * abs(boundary) + ATOL
            must = set(np.nonzero(oracle_scores > boundary + tol)[0].tolist())
            may = set(np.nonzero(oracle_scores >= boundary - tol)[0].tolist())
            got = set(idx.tolist())
            assert must <= got <= may, "selection disagrees with the oracle beyond the tolerance band"
            gap = oracle_scores[order[M - 1]] - oracle_scores[order[M]]
            if gap > 2 * tol or exact_sets:
                assert got == set(ref_idx.tolist()), "selected set differs from the oracle's"
        else:
            assert set(idx.tolist()) == set(ref_idx.tolist())
    return idx
