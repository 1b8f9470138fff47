"""GPU parity: libppow (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Sizes are ones the oracle finishes in seconds and still
span several 256-lane x 128-bit tiles plus ragged heads and tails."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_14978_amd as ppow
from workloads import WORKLOADS, generate

from parity import (ATOL_DIVERGENCE, RTOL, assert_close, check_selection, compare, compare_advantage,
                    compare_group_best, dtype_name,
                    run_gpu, run_oracle)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _to_dev(d):
    return {k: (None if v is None else v.to(DEV)) for k, v in d.items()}


def _random_inputs(B, K, V, dtype, seed, sigma=0.7, greedy=False, scale=3.0):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn(B, K, V, generator=g) * scale
    b = a + torch.randn(B, K, V, generator=g) * sigma
    a, b = a.to(dtype), b.to(dtype)
    tok = torch.randint(0, V, (B, K), generator=g, dtype=torch.int32)
    u = torch.rand(B, K, generator=g)
    d = {"target_logits": a, "draft_logits": b, "draft_tokens": tok, "uniforms": None if greedy else u}
    return _to_dev(d)


def _keep_decisions_clear(d, ref, verify):
    """Random test inputs carry no margins: nudge uniforms that sit within 1e-3 of alpha."""
    if verify == "greedy":
        return d, ref, False
    u = d["uniforms"].cpu().numpy()
    close = np.abs(u.astype(np.float64) - ref.accept_prob) < 1e-3
    if close.any():
        u = np.where(close, np.where(ref.accept_prob > 0.5, 0.0, 1.0), u).astype(np.float32)
        d = dict(d, uniforms=torch.from_numpy(u).to(DEV))
        return d, None, True
    return d, ref, False


def _check(d, V, *, cost_ratio=0.05, verify="rejection", expected_accept=False, M=None, **kw):
    dname = dtype_name(d["target_logits"])
    ref = run_oracle(d, cost_ratio=cost_ratio, verify=verify, expected_accept=expected_accept, **kw)
    d, ref2, changed = _keep_decisions_clear(d, ref, verify)
    if changed:
        ref = run_oracle(d, cost_ratio=cost_ratio, verify=verify, expected_accept=expected_accept, **kw)
    gpu = run_gpu(d, cost_ratio=cost_ratio, verify=verify, expected_accept=expected_accept, **kw)
    compare(gpu, ref, dname, V, expected_accept)
    if M:
        check_selection(gpu.adaw_score, M, ref.adaw_score, RTOL[dname])
    return gpu, ref


# ---- the benchmark's workloads at oracle-sized window counts -------------------------------

@pytest.mark.parametrize("name,B", [("tiny_f32", 32), ("greedy_bf16_32k", 96),
                                    ("rejection_bf16_128k", 40), ("twopass_f32_152k", 24),
                                    ("stream_bf16_128k", 24)])
def test_workload_matches_oracle(name, B):
    w = WORKLOADS[name].scaled(B)
    d = generate(w, device=DEV)
    ref = run_oracle(d, cost_ratio=w.cost_ratio, verify=w.verify, expected_accept=w.expected_accept)
    gpu = run_gpu(d, cost_ratio=w.cost_ratio, verify=w.verify, expected_accept=w.expected_accept)
    compare(gpu, ref, w.dtype, w.V, w.expected_accept)
    check_selection(gpu.adaw_score, w.M, ref.adaw_score, RTOL[w.dtype])
    assert 0 < ref.accepted_len.mean() < w.K        # the case exercises truncation


# ---- ragged shapes: heads, tails, fewer chunks than lanes ----------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [2, 3, 7, 8, 9, 31, 257, 1000, 1001, 1023, 2049, 4099, 8200, 20011])
def test_ragged_vocabulary_sizes(V, dtype):
    d = _random_inputs(5, 3, V, dtype, seed=V)
    _check(d, V, M=2)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("expected_accept", [False, True])
def test_rows_of_two_million_logits(dtype, expected_accept):
    """Rows far longer than any benchmark vocabulary (and not a multiple of the 128-bit chunk):
    thousands of chunks per lane, and more than any set of cooperating workgroups keeps on chip."""
    V = 2_000_003
    d = _random_inputs(2, 2, V, dtype, seed=77, sigma=0.5)
    _check(d, V, expected_accept=expected_accept, M=1)


@pytest.mark.parametrize("dtype,V", [(torch.float32, 1030), (torch.bfloat16, 2051), (torch.float32, 128)])
def test_more_rows_than_resident_workgroups(dtype, V):
    """Several times more row pairs than the device holds workgroups at once, also when the same
    buffers are used again: every row is written by every call (outputs start out poisoned)."""
    B, K = 2300, 5
    d = _random_inputs(B, K, V, dtype, seed=V, sigma=0.6)
    gpu, ref = _check(d, V, M=100)
    assert ppow.last_row_kernel() == "row"
    # the same call again into outputs that hold NaN: a row nobody claimed would keep it
    buf = ppow.ScoreBuffers(B, K, V, ppow.PPOW_BF16 if dtype == torch.bfloat16 else ppow.PPOW_F32, DEV,
                            ("kl", "confidence"))
    for _ in range(3):
        buf.kl.fill_(float("nan"))
        buf.adaw_score.fill_(float("nan"))
        ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
                                cost_ratio=0.05, buffers=buf)
        torch.cuda.synchronize()
        assert torch.equal(buf.kl, gpu.kl) and torch.equal(buf.adaw_score, gpu.adaw_score)


@pytest.mark.parametrize("K", [1, 2, 5, 16, 17, 33, 64])
def test_window_lengths(K):
    d = _random_inputs(9, K, 515, torch.float32, seed=100 + K, sigma=0.3)
    gpu, ref = _check(d, 515, M=3)
    assert ref.accepted_len.max() <= K


def test_empty_batch_is_a_noop():
    d = _random_inputs(1, 4, 64, torch.float32, seed=1)
    empty = {k: (None if v is None else v[:0].contiguous()) for k, v in d.items()}
    out = ppow.ppow_score_windows(empty["draft_logits"], empty["target_logits"],
                                  empty["draft_tokens"], empty["uniforms"], cost_ratio=0.1)
    torch.cuda.synchronize()
    assert out.accepted_len.numel() == 0


# ---- degenerate cases of the method ----------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_identical_logits_give_exact_zero_divergence_and_full_acceptance(dtype):
    d = _random_inputs(6, 8, 5003, dtype, seed=7)
    d["draft_logits"] = d["target_logits"].clone()
    d["uniforms"] = torch.ones_like(d["uniforms"])            # u = 1 still accepts: alpha = 1
    gpu = run_gpu(d, cost_ratio=0.03, verify="rejection")
    assert torch.all(gpu.kl == 0) and torch.all(gpu.adaw_score == 0)
    assert torch.all(gpu.accept_prob == 1) and torch.all(gpu.accepted_len == 8)
    ref = run_oracle(d, cost_ratio=0.03, verify="rejection")
    compare(gpu, ref, dtype_name(d["target_logits"]), 5003)


def test_mismatch_at_position_j_truncates_to_j_greedy():
    K, V = 8, 3001
    d = _random_inputs(K + 1, K, V, torch.bfloat16, seed=11, greedy=True)
    ystar = d["target_logits"].float().argmax(-1).to(torch.int32)
    tok = ystar.clone()
    for j in range(K):
        tok[j, j] = (ystar[j, j] + 1) % V
    d["draft_tokens"] = tok.contiguous()
    gpu, ref = _check(d, V, verify="greedy")
    assert gpu.accepted_len.cpu().tolist() == list(range(K)) + [K]


def test_argmax_ties_take_the_lowest_index():
    V = 4096 + 5
    a = torch.zeros(4, 2, V)
    a[0, 0, [9, 700, 4100]] = 5.0           # tie across lanes and chunks
    a[0, 1, [4100, 4099]] = 5.0             # tie inside the ragged tail
    a[1, 0, [0, 1]] = 5.0
    a[1, 1, [2047, 2048]] = 5.0
    a[2, :, 300] = 5.0
    a[3, :, V - 1] = 5.0
    b = a + 0.1 * torch.randn(a.shape, generator=torch.Generator().manual_seed(3))
    first = torch.tensor([[9, 4099], [0, 2047], [300, 300], [V - 1, V - 1]], dtype=torch.int32)
    for tok, expect in ((first, [2, 2, 2, 2]),
                        (torch.tensor([[700, 4100], [1, 2048], [300, 300], [V - 1, V - 1]],
                                      dtype=torch.int32), [0, 0, 2, 2])):
        d = _to_dev({"target_logits": a, "draft_logits": b, "draft_tokens": tok, "uniforms": None})
        gpu, ref = _check(d, V, verify="greedy")
        assert gpu.accepted_len.cpu().tolist() == expect


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_argmax_ties_in_the_second_pass_kernel(dtype):
    """Equal maxima in different lanes, register / LDS chunks, members of a cluster and in the
    ragged tail: the first index wins on the path that keeps the row on chip as well."""
    V = 60001                               # fp32: two members; rows are not 16-byte aligned
    a = torch.zeros(4, 2, V)
    a[0, 0, [12345, 12346, 50000]] = 5.0    # inside one chunk, and in the other member
    a[0, 1, [40000, 59999, 60000]] = 5.0    # LDS part of member 0 / member 1, and the tail
    a[1, 0, [0, 1, 2, 3]] = 5.0             # the head, before the first aligned chunk
    a[1, 1, [30001, 30000]] = 5.0           # around the member boundary
    a[2, :, 2048 * 9 + 5] = 5.0
    a[3, :, V - 1] = 5.0
    b = a + 0.1 * torch.randn(a.shape, generator=torch.Generator().manual_seed(4))
    first = torch.tensor([[12345, 40000], [0, 30000], [2048 * 9 + 5] * 2, [V - 1, V - 1]], dtype=torch.int32)
    later = torch.tensor([[12346, 59999], [1, 30001], [2048 * 9 + 5] * 2, [V - 1, V - 1]], dtype=torch.int32)
    for tok, expect in ((first, [2, 2, 2, 2]), (later, [0, 0, 2, 2])):
        d = _to_dev({"target_logits": a.to(dtype), "draft_logits": b.to(dtype), "draft_tokens": tok,
                     "uniforms": None})
        gpu, ref = _check(d, V, verify="greedy", expected_accept=True)
        assert ppow.last_row_kernel() == "cluster"
        assert gpu.accepted_len.cpu().tolist() == expect


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_reference_rescaling_on_monotone_and_wide_range_rows(dtype):
    """Rows whose maximum keeps growing along the vocabulary force the running
    reference to be rebased many times; very negative logits must vanish cleanly."""
    B, K, V = 4, 3, 6000
    ramp = torch.linspace(-300.0, 300.0, V)
    a = torch.stack([ramp, ramp.flip(0), ramp * 0.2, torch.full((V,), -1000.0)])
    a = a[:, None, :].repeat(1, K, 1).contiguous()
    a[3, :, 17] = 900.0
    a[3, :, 4000] = 899.0
    g = torch.Generator().manual_seed(5)
    b = a * 0.97 + torch.randn(B, K, V, generator=g)
    tok = a.argmax(-1).to(torch.int32)
    tok[:, 1] = (tok[:, 1] + 3) % V
    d = _to_dev({"target_logits": a.to(dtype), "draft_logits": b.to(dtype), "draft_tokens": tok,
                 "uniforms": torch.full((B, K), 0.5)})
    _check(d, V)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_second_pass_on_rows_whose_reference_keeps_moving(dtype):
    """The on-chip second pass of fp32 rows rescales exponentials it kept from the first pass;
    a ramp along the vocabulary moves every lane's reference at every chunk, in the register
    part, in the LDS part and at the ragged tail (V = 18001: rows are not 16-byte aligned)."""
    B, K, V = 3, 2, 18001
    ramp = torch.linspace(-300.0, 300.0, V)
    a = torch.stack([ramp, ramp.flip(0), ramp * 0.05])
    a = a[:, None, :].repeat(1, K, 1).contiguous()
    g = torch.Generator().manual_seed(11)
    b = a * 0.97 + torch.randn(B, K, V, generator=g)
    tok = a.argmax(-1).to(torch.int32)
    tok[:, 1] = (tok[:, 1] + 5) % V
    d = _to_dev({"target_logits": a.to(dtype), "draft_logits": b.to(dtype), "draft_tokens": tok,
                 "uniforms": torch.full((B, K), 0.5)})
    _check(d, V, expected_accept=True)
    assert ppow.last_row_kernel() == "cluster"


@pytest.mark.parametrize("seed", range(24))
def test_random_option_combinations(seed):
    """Seeded random shapes and option sets, second pass and policy terms included, down to
    vocabularies shorter than one 16-byte chunk."""
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([2, 3, 5, 8, 13, 64, 127, 1000, 2051, 5000, 12289, 33001, 70001]))
    K = int(rng.choice([1, 2, 3, 4, 7, 10, 16, 33]))
    B = int(rng.integers(1, 7)) * (2 if K <= 4 else 1)
    dtype = torch.float32 if rng.random() < 0.5 else torch.bfloat16
    greedy = bool(rng.random() < 0.4)
    group = int(rng.choice([0, 1, 2])) if B % 2 == 0 else int(rng.choice([0, 1]))
    d = _random_inputs(B, K, V, dtype, seed=seed, sigma=float(rng.choice([0.2, 1.0, 3.0])), greedy=greedy,
                       scale=float(rng.choice([0.5, 3.0, 8.0])))
    if greedy:                      # let some prefixes survive
        d["draft_tokens"] = torch.where(torch.rand(B, K, device=DEV) < 0.6,
                                        d["target_logits"].float().argmax(-1).to(torch.int32),
                                        d["draft_tokens"]).contiguous()
    kw = {}
    if group:
        kw["rollout_group"] = group
    _check(d, V, verify="greedy" if greedy else "rejection",
           expected_accept=bool(rng.random() < 0.6), policy_terms=bool(rng.random() < 0.5),
           cost_ratio=float(rng.choice([0.01, 0.03, 0.5])), **kw)


def test_uniform_target_has_zero_confidence():
    V = 2048
    a = torch.full((2, 2, V), 1.5)
    b = torch.randn(2, 2, V, generator=torch.Generator().manual_seed(1)) * 2
    d = _to_dev({"target_logits": a, "draft_logits": b, "draft_tokens": torch.zeros(2, 2, dtype=torch.int32),
                 "uniforms": torch.full((2, 2), 0.5)})
    gpu = run_gpu(d, cost_ratio=0.1, verify="rejection")
    assert float(gpu.confidence.abs().max()) < 1e-6 and float(gpu.adaw_score.abs().max()) < 1e-5


def test_proximity_reward_and_reference_logprob():
    V, K = 512, 2
    a = torch.zeros(4, K, V)
    a[:, :, 0] = 4.0
    a[0, 0, 1], a[0, 1, 1] = 3.75, 3.76      # gap 0.49 -> eta
    a[1, 0, 1], a[1, 1, 1] = 3.75, 3.74      # gap 0.51 -> 0
    a[2, :, 1] = 3.9                         # small gap but k >= 1
    a[3, 0, 1], a[3, 1, 1] = 3.5, 4.0 - 2.0 ** -10   # gap 0.5 + 2^-10: just outside
    b = a.clone()
    b[:, :, 1] += 3.0
    tok = torch.ones(4, K, dtype=torch.int32)
    u = torch.full((4, K), 0.999)
    u[2, 0] = 0.0
    d = _to_dev({"target_logits": a, "draft_logits": b, "draft_tokens": tok, "uniforms": u})
    gpu, ref = _check(d, V, prox_eta=0.75)
    assert gpu.accepted_len.cpu().tolist() == [0, 0, 1, 0]
    assert gpu.r_proximity.cpu().tolist() == [0.75, 0.0, 0.0, 0.0]
    # with a caller-supplied reference log-probability: delta = ref - sum_t log P_t(tok_t)
    ref_lp = torch.tensor([-0.3, -2.0, -1.0, -0.9]).to(DEV)
    gpu, ref = _check(d, V, prox_eta=0.75, ref_logprob=ref_lp)
    assert float(np.abs(ref.delta - 0.5).min()) > 1e-3


def test_expected_accept_pass_small_and_ragged():
    for V, dtype in ((1000, torch.float32), (4099, torch.bfloat16), (33000, torch.float32)):
        d = _random_inputs(4, 3, V, dtype, seed=V + 1, sigma=1.0)
        gpu, ref = _check(d, V, expected_accept=True)
        kl = gpu.kl.double().cpu().numpy()
        ea = gpu.expected_accept.double().cpu().numpy()
        assert np.all(ea >= 1.0 - np.sqrt(0.5 * kl) - 1e-5)          # Pinsker (Appendix B.1)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [9, 1001, 4099, 40000])
def test_policy_terms_reverse_kl_and_alignment(V, dtype):
    d = _random_inputs(6, 4, V, dtype, seed=3 * V + 1, sigma=1.0)
    gpu, ref = _check(d, V, policy_terms=True)
    assert gpu.reverse_kl is not None and float(gpu.reverse_kl.min()) >= 0
    # the same windows with the expected-acceptance pass on top (cluster kernel variant)
    _check(d, V, policy_terms=True, expected_accept=True)


def test_policy_terms_vanish_for_identical_rows():
    d = _random_inputs(3, 4, 3000, torch.bfloat16, seed=5)
    d["draft_logits"] = d["target_logits"].clone()
    gpu = run_gpu(d, cost_ratio=0.05, verify="rejection", policy_terms=True)
    assert torch.all(gpu.reverse_kl == 0) and torch.all(gpu.alignment == 0)
    assert torch.all(gpu.reverse_kl_mean == 0) and torch.all(gpu.alignment_mean == 0)


@pytest.mark.parametrize("group", [1, 2, 8])
def test_group_relative_advantage(group):
    w = WORKLOADS["tiny_f32"].scaled(32)
    d = generate(w, device=DEV)
    ref = run_oracle(d, cost_ratio=w.cost_ratio, verify=w.verify)
    gpu = run_gpu(d, cost_ratio=w.cost_ratio, verify=w.verify, rollout_group=group, adv_delta=1e-4)
    compare(gpu, ref, w.dtype, w.V)
    compare_advantage(gpu, ref, group, 1e-4, RTOL[w.dtype])
    compare_group_best(gpu, ref, group)
    adv = gpu.advantage.cpu().view(-1, group)
    assert float(adv.sum(-1).abs().max()) < 1e-4           # zero mean inside every group


@pytest.mark.parametrize("group", [3, 5, 6, 7, 8])
def test_group_advantage_of_equal_rewards_is_exactly_zero(group):
    """Rewards that are equal across a rollout group (every window fully accepted, or every
    window rejected at once) have advantage 0 by definition (Section 4.1); with the default
    delta = 1e-6 any rounding residue of the mean would be blown up to ~0.1.  Mixed groups are
    compared with the oracle at the same delta."""
    K, V, groups = 3, 257, 6
    B = group * groups
    d = _random_inputs(B, K, V, torch.float32, seed=90 + group, greedy=True)
    ystar = d["target_logits"].argmax(-1).to(torch.int32)
    far = d["target_logits"].argmin(-1).to(torch.int32)   # a gap far above eps: no proximity reward
    tok = ystar.clone()                                   # groups 0, 1: all accepted (k = K)
    tok[2 * group:4 * group, 0] = far[2 * group:4 * group, 0]               # groups 2, 3: k = 0
    for b in range(4 * group, B):                         # groups 4, 5: k cycles through 0..K
        k = b % (K + 1)
        if k < K:
            tok[b, k] = far[b, k]
    d["draft_tokens"] = tok.contiguous()
    for gamma in (0.03, 0.12, 1.0 / 3.0):
        ref = run_oracle(d, cost_ratio=gamma, verify="greedy")
        gpu = run_gpu(d, cost_ratio=gamma, verify="greedy", rollout_group=group)   # delta = 1e-6
        compare(gpu, ref, "f32", V)
        adv = gpu.advantage.cpu().view(groups, group)
        assert torch.all(adv[:4] == 0), adv[:4]
        compare_advantage(gpu, ref, group, 1e-6, RTOL["f32"])
        compare_group_best(gpu, ref, group)


def test_group_best_with_ties_takes_the_first_candidate():
    K, V = 4, 300
    d = _random_inputs(12, K, V, torch.float32, seed=21, greedy=True)
    ystar = d["target_logits"].argmax(-1).to(torch.int32)
    tok = ystar.clone()
    lens = [0, 2, 2, 1, 4, 4, 3, 4, 1, 1, 0, 1]          # groups of 4: best 2@1, 4@0, 1@0
    for b, k in enumerate(lens):
        if k < K:
            tok[b, k] = (ystar[b, k] + 1) % V
    d["draft_tokens"] = tok.contiguous()
    gpu = run_gpu(d, cost_ratio=0.1, verify="greedy", rollout_group=4)
    assert gpu.accepted_len.cpu().tolist() == lens
    assert gpu.group_best_len.cpu().tolist() == [2, 4, 1]
    assert gpu.group_best_index.cpu().tolist() == [1, 0, 0]


# ---- sequence-mode ADAW (Algorithm 1) ---------------------------------------------------------

def _sequence_inputs(N, T, V, dtype, seed, sigma=0.8):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn(N, T, V, generator=g) * 3.0
    sig = torch.rand(N, T, 1, generator=g) * sigma * 2
    b = a + torch.randn(N, T, V, generator=g) * sig
    return a.to(dtype).to(DEV), b.to(dtype).to(DEV), torch.rand(N, generator=g).to(DEV)


@pytest.mark.parametrize("N,T,V,K,dtype", [(3, 12, 1001, 4, torch.float32), (2, 40, 4099, 10, torch.bfloat16),
                                           (5, 7, 300, 7, torch.float32), (4, 9, 515, 1, torch.bfloat16),
                                           (1, 300, 2000, 64, torch.float32),
                                           (1, 8300, 64, 5, torch.float32)])
def test_sequence_mode_matches_oracle(N, T, V, K, dtype):
    a, b, u = _sequence_inputs(N, T, V, dtype, seed=N * 1000 + T)
    out = ppow.ppow_adaw_sequence(b, a, K, u)
    torch.cuda.synchronize()
    v_ref, s_ref = oracle.adaw_sequence(b.cpu(), a.cpu(), K)
    rtol = RTOL[dtype_name(a)]
    assert_close("criticality", out.criticality.cpu(), v_ref, rtol, ATOL_DIVERGENCE)
    assert_close("window_score", out.window_score.cpu(), s_ref, rtol, ATOL_DIVERGENCE)
    # the sampler is exact on the scores the GPU itself produced ...
    s_gpu = out.window_score.cpu().numpy().astype(np.float64)
    picks = oracle.sample_starts(s_gpu, u.cpu().numpy().astype(np.float64))
    assert np.array_equal(out.sampled_start.cpu().numpy(), picks)
    # ... and agrees with the oracle end to end wherever the draw is not within the float
    # tolerance of a boundary of the cumulative distribution
    c = np.cumsum(s_ref, axis=1)
    thr = u.cpu().numpy().astype(np.float64) * c[:, -1]
    clear = np.abs(c - thr[:, None]).min(1) > 10 * rtol * c[:, -1]
    ref_picks = oracle.sample_starts(s_ref, u.cpu().numpy().astype(np.float64))
    assert np.array_equal(out.sampled_start.cpu().numpy()[clear], ref_picks[clear])
    # scoring the overlapping windows one by one gives the same scores (K x the bytes)
    if T <= 40:
        W = T - K + 1
        wa = torch.stack([a[n, j:j + K] for n in range(N) for j in range(W)]).contiguous()
        wb = torch.stack([b[n, j:j + K] for n in range(N) for j in range(W)]).contiguous()
        d = {"target_logits": wa, "draft_logits": wb, "uniforms": torch.ones(N * W, K, device=DEV),
             "draft_tokens": torch.zeros(N * W, K, dtype=torch.int32, device=DEV)}
        win = run_gpu(d, cost_ratio=0.1, verify="rejection")
        assert_close("window mode", win.adaw_score.cpu(), out.window_score.cpu().reshape(-1), 1e-5)


@pytest.mark.parametrize("rho", [0.0, 0.2, 0.4, 0.6, 1.0])
def test_sequence_mode_curriculum_mixes_adaw_and_uniform_starts(rho):
    """Hard-window curriculum (Appendix A.3, Table 5): the start of sequence n is ADAW-selected
    iff its mixing draw is below rho; the decision and the start are the oracle's on the GPU's
    own scores, for many sequences (short ones: one row of logits is enough to score)."""
    N, T, V, K = 96, 70, 64, 5
    a, b, u = _sequence_inputs(N, T, V, torch.float32, seed=4242)
    g = torch.Generator().manual_seed(int(rho * 100) + 1)
    mix = torch.rand(N, generator=g).to(DEV)
    mix[:4] = torch.tensor([0.2, 0.4, 0.6, 0.0])              # draws that sit on the schedule's values
    out = ppow.ppow_adaw_sequence(b, a, K, u, adaw_fraction=rho, mix_uniforms=mix)
    torch.cuda.synchronize()
    s_gpu = out.window_score.cpu().numpy().astype(np.float64)
    u64, m64 = u.cpu().numpy().astype(np.float64), mix.cpu().numpy().astype(np.float64)
    rho32 = float(np.float32(rho))                             # the fraction crosses the ABI as a float
    picks = oracle.sample_starts_curriculum(s_gpu, u64, m64, rho32)
    assert np.array_equal(out.sampled_start.cpu().numpy(), picks)
    adaw = m64 < rho32
    W = T - K + 1
    assert np.array_equal(picks[~adaw], np.minimum(np.floor(u64[~adaw] * W), W - 1).astype(np.int64))
    if 0 < rho < 1:
        assert adaw.any() and (~adaw).any()
        # the two kinds of start really differ on these inputs
        assert (oracle.sample_starts(s_gpu, u64) != picks).any()
    if rho == 1.0:     # the draws are not needed, and not looked at
        plain = ppow.ppow_adaw_sequence(b, a, K, u)
        torch.cuda.synchronize()
        assert torch.equal(plain.sampled_start, out.sampled_start)


def test_sequence_mode_degenerate_scores_sample_uniformly():
    a, _, _ = _sequence_inputs(2, 10, 200, torch.float32, seed=9)
    u = torch.tensor([0.0, 0.73], device=DEV)
    out = ppow.ppow_adaw_sequence(a.clone(), a, 3, u)          # identical rows: every score is zero
    torch.cuda.synchronize()
    assert torch.all(out.window_score == 0)
    assert out.sampled_start.cpu().tolist() == [0, int(0.73 * 8)]
    no_sampling = ppow.ppow_adaw_sequence(a.clone(), a, 3)
    torch.cuda.synchronize()
    assert no_sampling.sampled_start is None and torch.all(no_sampling.criticality == 0)


def test_second_pass_rows_longer_than_one_slice_and_many_rows_per_cluster():
    """More row pairs than clusters, and rows long enough to be split over several members."""
    for dtype, V in ((torch.float32, 50021), (torch.bfloat16, 70003)):
        d = _random_inputs(150, 4, V, dtype, seed=V, sigma=0.8)
        _check(d, V, expected_accept=True, M=20)
        assert ppow.last_row_kernel() == "cluster"          # the LDS-resident path really ran
        _check(d, V, M=20)
        assert ppow.last_row_kernel() == "row"
    # greedy verification together with the second pass
    d = _random_inputs(40, 5, 9001, torch.bfloat16, seed=77, greedy=True)
    d["draft_tokens"] = torch.where(torch.rand(40, 5, device=DEV) < 0.7,
                                    d["target_logits"].float().argmax(-1).to(torch.int32),
                                    d["draft_tokens"]).contiguous()
    gpu, ref = _check(d, 9001, verify="greedy", expected_accept=True)
    assert 0 < ref.accepted_len.mean() < 5


def test_expired_wait_of_the_on_chip_second_pass_marks_every_window():
    """The give-up path of the cluster kernel, reached by shrinking its bounded wait to a single
    look from the host: every kernel still ends normally, the status word is set and every
    window of the call is reported with accepted_len = -3, zero rewards and score 0."""
    V = 50021
    d = _random_inputs(150, 4, V, torch.float32, seed=5, sigma=0.8)
    L = ppow.lib()
    L.ppow_debug_cluster_wait_limit(1)
    try:
        out = ppow.ppow_score_windows(
            d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
            cost_ratio=0.05, flags=ppow.PPOW_FLAG_EXPECTED_ACCEPT, optional=("expected_accept",))
        assert ppow.last_row_kernel() == "cluster"
        torch.cuda.synchronize()
    finally:
        L.ppow_debug_cluster_wait_limit(0)
    if out.status() != 0:          # with one look some member practically always misses a partner
        assert torch.all(out.accepted_len == -3)
        assert torch.all(out.r_speedup == 0) and torch.all(out.r_proximity == 0)
        assert torch.all(out.adaw_score == 0)
    # the next call, with the default limit, is unaffected by what the expired one left behind
    _check(d, V, expected_accept=True, M=20)
    assert ppow.last_row_kernel() == "cluster"


@pytest.mark.parametrize("expected_accept", [False, True])
def test_tokens_outside_the_vocabulary_mark_their_window_and_nothing_else(expected_accept):
    """The device, not the host, sees the drafted tokens: an out-of-range one must not be used
    as an address (the kernel substitutes element 0) and its window reports accepted_len = -1."""
    B, K, V = 12, 3, 5003
    d = _random_inputs(B, K, V, torch.float32, seed=31)
    good = dict(d)
    tok = d["draft_tokens"].clone()
    bad_windows = {1: (0, V), 4: (2, -1), 7: (1, 2 ** 30), 11: (0, -2 ** 31)}
    for b, (t, value) in bad_windows.items():
        tok[b, t] = value
    d["draft_tokens"] = tok
    gpu = run_gpu(d, cost_ratio=0.05, verify="rejection", expected_accept=expected_accept)
    ref = run_oracle(good, cost_ratio=0.05, verify="rejection", expected_accept=expected_accept)
    k = gpu.accepted_len.cpu().numpy()
    ok = np.array([b not in bad_windows for b in range(B)])
    assert np.all(k[~ok] == -1) and np.array_equal(k[ok], ref.accepted_len[ok])
    assert np.all(gpu.r_speedup.cpu().numpy()[~ok] == 0) and np.all(gpu.r_proximity.cpu().numpy()[~ok] == 0)
    np.testing.assert_allclose(gpu.r_speedup.cpu().numpy()[ok], ref.r_speedup[ok], rtol=1e-6)
    np.testing.assert_allclose(gpu.adaw_score.cpu().numpy(), ref.adaw_score, rtol=RTOL["f32"],
                               atol=ATOL_DIVERGENCE)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("expected_accept", [False, True])
def test_windows_with_non_finite_logits_are_marked(dtype, expected_accept):
    """Finite logits are a precondition; a NaN or an infinity must still be visible in the
    result (accepted_len = -2, no reward, score 0) and must not disturb other windows."""
    B, K, V = 10, 3, 9001
    d = _random_inputs(B, K, V, dtype, seed=61)
    clean = {k: (None if v is None else v.clone()) for k, v in d.items()}
    d["target_logits"][2, 1, 4000] = float("nan")
    d["draft_logits"][5, 0, 17] = float("inf")
    d["target_logits"][8, 2, V - 1] = float("-inf")
    d["draft_logits"][9, 2, 0] = float("-inf")
    bad = [2, 5, 8, 9]
    gpu = run_gpu(d, cost_ratio=0.05, verify="rejection", expected_accept=expected_accept)
    ref = run_oracle(clean, cost_ratio=0.05, verify="rejection", expected_accept=expected_accept)
    k = gpu.accepted_len.cpu().numpy()
    ok = np.array([b not in bad for b in range(B)])
    assert np.all(k[~ok] == -2) and np.array_equal(k[ok], ref.accepted_len[ok])
    for name in ("r_speedup", "r_proximity", "adaw_score"):
        assert np.all(getattr(gpu, name).cpu().numpy()[~ok] == 0), name
    np.testing.assert_allclose(gpu.adaw_score.cpu().numpy()[ok], ref.adaw_score[ok],
                               rtol=RTOL[dtype_name(d["target_logits"])], atol=ATOL_DIVERGENCE)


def test_calls_on_a_side_stream_and_back_to_back_calls_sharing_a_workspace():
    """The library enqueues on the stream it is given; calls that share a workspace on one
    stream run one after another and must not disturb each other."""
    w = WORKLOADS["tiny_f32"].scaled(32)
    d = generate(w, device=DEV)
    ref = run_oracle(d, cost_ratio=w.cost_ratio, verify=w.verify, expected_accept=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT
    opt = ("delta", "kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok",
           "expected_accept")
    with torch.cuda.stream(side):
        bufs = ppow.ScoreBuffers(w.B, w.K, w.V, ppow.PPOW_F32, DEV, opt, flags)
        halves = [bufs.window_slice(0, 16), bufs.window_slice(16, 32)]
        for rep in range(3):                      # same workspace, alternating halves
            for h, (lo, hi) in zip(halves, ((0, 16), (16, 32))):
                ppow.ppow_score_windows(d["draft_logits"][lo:hi], d["target_logits"][lo:hi],
                                        d["draft_tokens"][lo:hi], d["uniforms"][lo:hi],
                                        cost_ratio=w.cost_ratio, flags=flags, buffers=h, stream=side)
        sel = ppow.ppow_select_windows(bufs.adaw_score, w.M, stream=side)
    side.synchronize()
    compare(bufs, ref, w.dtype, w.V, True)
    assert np.array_equal(sel.indices.cpu().numpy(),
                          oracle.select_windows(bufs.adaw_score.cpu().numpy().astype(np.float64), w.M))


def test_second_pass_calls_on_two_streams_at_once():
    """Each on-chip second-pass kernel needs the whole GPU, so the library chains such launches
    across streams; calls issued back to back on two streams must both come out right."""
    V, K = 50021, 4
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT
    opt = ("kl", "expected_accept", "accept_prob")
    cases = []
    for seed in (51, 52):
        d = _random_inputs(600, K, V, torch.float32, seed=seed, sigma=0.8)
        ref = run_oracle(d, cost_ratio=0.05, verify="rejection", expected_accept=True)
        d, _, changed = _keep_decisions_clear(d, ref, "rejection")
        if changed:
            ref = run_oracle(d, cost_ratio=0.05, verify="rejection", expected_accept=True)
        cases.append((d, ref, ppow.ScoreBuffers(600, K, V, ppow.PPOW_F32, DEV, opt, flags), torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(3):
        for d, ref, bufs, stream in cases:
            ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
                                    cost_ratio=0.05, flags=flags, buffers=bufs, stream=stream)
            assert ppow.last_row_kernel() == "cluster"
    torch.cuda.synchronize()
    for d, ref, bufs, stream in cases:
        assert bufs.status() == 0
        compare(bufs, ref, "f32", V, True)


def test_scoring_and_selection_replay_from_a_hip_graph():
    """The single-pass path allocates nothing and records no memset node, so it can be captured
    once and replayed; every replay must reproduce the eager result bit for bit, with eager work
    and synchronisations in between."""
    w = WORKLOADS["greedy_bf16_32k"].scaled(64)
    d = generate(w, device=DEV)
    bufs = ppow.ScoreBuffers(w.B, w.K, w.V, ppow.PPOW_BF16, DEV, ("delta", "kl"))
    sel = ppow.SelectBuffers(w.B, w.M, DEV)

    def step():
        ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"], None,
                                cost_ratio=w.cost_ratio, verify=ppow.PPOW_VERIFY_GREEDY, buffers=bufs)
        ppow.ppow_select_windows(bufs.adaw_score, w.M, buffers=sel)

    step()
    torch.cuda.synchronize()
    eager = {n: getattr(bufs, n).clone() for n in ("accepted_len", "r_speedup", "adaw_score", "kl")}
    eager_idx = sel.indices.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    for replay in range(3):
        for t in (bufs.accepted_len, bufs.r_speedup, bufs.adaw_score, bufs.kl, sel.indices):
            t.zero_()                                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, ref in eager.items():
            assert torch.equal(getattr(bufs, n), ref), (replay, n)
        assert torch.equal(sel.indices, eager_idx), replay


def test_second_pass_can_be_captured_into_a_hip_graph():
    """A cooperative launch cannot be recorded, so under capture the second pass runs from
    memory; the replays must agree with the oracle like the eager (on-chip) result does."""
    V = 30011
    d = _random_inputs(24, 3, V, torch.float32, seed=41, sigma=1.0)
    ref = run_oracle(d, cost_ratio=0.05, verify="rejection", expected_accept=True)
    d, _, changed = _keep_decisions_clear(d, ref, "rejection")
    if changed:
        ref = run_oracle(d, cost_ratio=0.05, verify="rejection", expected_accept=True)
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT
    opt = ("delta", "kl", "confidence", "accept_prob", "logp_target_tok", "logp_draft_tok", "expected_accept")
    bufs = ppow.ScoreBuffers(24, 3, V, ppow.PPOW_F32, DEV, opt, flags)

    def step():
        ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
                                cost_ratio=0.05, flags=flags, buffers=bufs)

    step()
    torch.cuda.synchronize()
    assert ppow.last_row_kernel() == "cluster"
    compare(bufs, ref, "f32", V, True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    assert ppow.last_row_kernel() == "row"
    for replay in range(3):
        for t in (bufs.accepted_len, bufs.adaw_score, bufs.expected_accept, bufs.kl):
            t.zero_()                                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        compare(bufs, ref, "f32", V, True)
        assert bufs.status() == 0


def test_results_are_bitwise_reproducible():
    w = WORKLOADS["rejection_bf16_128k"].scaled(16)
    d = generate(w, device=DEV)
    for extra in ({}, {"expected_accept": True, "policy_terms": True}):
        outs = [run_gpu(d, cost_ratio=w.cost_ratio, verify=w.verify, **extra) for _ in range(3)]
        names = ["accepted_len", "r_speedup", "r_proximity", "adaw_score", "delta", "kl"]
        names += ["expected_accept", "reverse_kl", "alignment"] if extra else []
        for o in outs[1:]:
            for name in names:
                assert torch.equal(getattr(o, name), getattr(outs[0], name)), name


# ---- selection -----------------------------------------------------------------------------

@pytest.mark.parametrize("B,M", [(1, 1), (2, 1), (7, 7), (100, 1), (100, 99), (1000, 8), (4096, 512),
                                 (16384, 2048), (65536, 8192), (65536, 1), (70001, 5000),
                                 (40000, 20000), (40000, 40000), (300000, 1024)])
def test_select_matches_full_sort(B, M):
    g = torch.Generator().manual_seed(B + M)
    s = torch.randn(B, generator=g)
    s[torch.randint(0, B, (max(1, B // 10),), generator=g)] = 0.25       # many exact ties
    if B > 50:
        s[[3, 17, 40]] = float(s.max()) + 1.0                                # ties at the top
        s[5] = -0.0
        s[6] = 0.0
    check_selection(s.to(DEV), M)


@pytest.mark.parametrize("seed", range(12))
def test_select_random_shapes_cover_every_kernel_and_sort_width(seed):
    """Seeded random (B, M): register-resident selection with 4 / 16 / 32 composites per thread,
    sorts of 2 / 4 / 8 composites per thread, slices with a ragged last one, and the general
    kernel; scores with heavy ties, negative values and a narrow range."""
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.choice([rng.integers(1, 5000), rng.integers(5000, 33000), rng.integers(33000, 200000)]))
    M = int(rng.choice([1, rng.integers(1, min(B, 2048) + 1), rng.integers(1, min(B, 8192) + 1),
                        rng.integers(1, B + 1)]))
    kind = seed % 3
    g = torch.Generator().manual_seed(seed)
    if kind == 0:
        s = torch.rand(B, generator=g) * 0.01 + 0.9                 # one exponent, crowded digits
    elif kind == 1:
        s = torch.randint(0, 7, (B,), generator=g).float() - 3.0    # seven distinct values: ties
    else:
        s = torch.randn(B, generator=g) * torch.rand(B, generator=g).pow(8) * 1e3   # wide range
    check_selection(s.to(DEV), M)


@pytest.mark.parametrize("B,M", [(30000, 3000), (100000, 4096), (49153, 2049), (32768, 8192),
                                 (32769, 1), (180000, 700), (50000, 50)])
def test_select_shapes_at_the_kernel_boundaries(B, M):
    g = torch.Generator().manual_seed(B ^ M)
    s = torch.rand(B, generator=g)
    s[torch.randint(0, B, (B // 7,), generator=g)] = 0.5
    check_selection(s.to(DEV), M)
    check_selection(torch.full((B,), 0.25, device=DEV), M)         # all equal: the M lowest indices


def test_select_tie_at_the_boundary_prefers_lower_indices():
    s = torch.zeros(5000)
    s[::7] = 1.0                                   # 715 ones; the rest tie at zero
    idx = check_selection(s.to(DEV), 1000)
    assert idx[:715].tolist() == list(range(0, 5000, 7))
    rest = [i for i in range(5000) if i % 7][:285]
    assert idx[715:].tolist() == rest
