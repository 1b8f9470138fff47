"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these re-types the oracle's own formula: each checks a printed value,
a closed form, an invariant, a brute-force enumeration, or a float64 library
routine on a special case, chosen so that a dropped term, a wrong sign or
index, or a transposed operand in the oracle fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _softmax64(x):
    return torch.softmax(torch.as_tensor(x, dtype=torch.float64), dim=-1).numpy()


def _rand_pair(rng, V, sigma=0.7, scale=3.0):
    a = rng.normal(0.0, scale, size=V)
    b = a + rng.normal(0.0, sigma, size=V)
    return a, b


def _score(a, b, tok, u=None, **kw):
    """a, b: [B, K, V] float64 values exactly representable in float32."""
    kw.setdefault("cost_ratio", 0.1)
    return oracle.score_windows(np.asarray(b, np.float32), np.asarray(a, np.float32), tok, u, **kw)


# ---- P1: the printed Cost-Aware Speedup Reward column (Table 6) -------------------------

def _table6():
    rows = []
    with open(os.path.join(GOLDEN, "table6_cost_aware_speedup.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, r = line.split()
                rows.append((int(k), float(r)))
    return rows


def test_speedup_reward_reproduces_table6():
    rows = _table6()
    assert [k for k, _ in rows] == [1, 2, 3, 4, 5, 6, 7]
    for k, printed in rows:
        assert round(oracle.speedup_reward(k, 0.1245), 2) == pytest.approx(printed, abs=1e-9)
    # Table 5's rounded gamma does not reproduce the column: guards against a
    # test that would pass for any gamma.
    assert any(round(oracle.speedup_reward(k, 0.12), 2) != printed for k, printed in rows)


def test_speedup_reward_bounds_and_monotone():
    for gamma in (0.03, 0.05, 0.12, 1.0):
        vals = [oracle.speedup_reward(k, gamma) for k in range(0, 65)]
        assert vals[0] == 0.0
        assert all(x < y for x, y in zip(vals, vals[1:]))      # strictly increasing in k
        assert all(v < 1.0 / gamma for v in vals)              # bounded by 1/gamma
    assert oracle.speedup_reward(3, 0.0) == 3.0                # zero drafting cost: raw k
    assert oracle.speedup_reward(1, 1.0) == 0.5


# ---- P2: identical draft and target ------------------------------------------------------

def test_identical_logits_zero_divergence_full_acceptance():
    rng = np.random.default_rng(1)
    B, K, V = 3, 5, 257
    a = rng.normal(0, 3, size=(B, K, V)).astype(np.float32)
    tok = rng.integers(0, V, size=(B, K))
    for u in (np.zeros((B, K)), np.ones((B, K)), rng.random((B, K))):
        r = oracle.score_windows(a.copy(), a, tok, u, cost_ratio=0.05,
                                 want=("kl", "accept_prob", "expected_accept", "reverse_kl",
                                       "alignment"))
        assert np.all(r.kl == 0.0) and np.all(r.reverse_kl == 0.0)
        assert np.all(r.adaw_score == 0.0)
        assert np.all(r.accept_prob == 1.0)
        assert np.all(r.alignment == 0.0)
        assert np.all(r.accepted_len == K)
        np.testing.assert_allclose(r.expected_accept, 1.0, rtol=0, atol=1e-12)
        np.testing.assert_allclose(r.r_speedup, K / (K * 0.05 + 1.0), rtol=1e-15)


# ---- P3: a mismatch at 0-based position j truncates acceptance to j ---------------------

@pytest.mark.parametrize("K", [1, 4, 7])
def test_greedy_first_mismatch_truncates(K):
    rng = np.random.default_rng(2)
    V = 64
    a = rng.normal(0, 2, size=(K + 1, K, V)).astype(np.float32)
    b = (a + rng.normal(0, 0.5, size=a.shape)).astype(np.float32)
    ystar = a.argmax(-1)
    tok = ystar.copy()
    for j in range(K):             # window j: only position j mismatches, later ones match
        tok[j, j] = (ystar[j, j] + 1) % V
    r = oracle.score_windows(b, a, tok, None, cost_ratio=0.1, verify=oracle.GREEDY)
    assert list(r.accepted_len) == list(range(K)) + [K]
    assert np.array_equal(r.argmax_target, ystar)


def test_rejection_first_failure_truncates_regardless_of_later_accepts():
    rng = np.random.default_rng(3)
    K, V = 6, 40
    a = rng.normal(0, 2, size=(K + 1, K, V)).astype(np.float32)
    b = (a + rng.normal(0, 1.0, size=a.shape)).astype(np.float32)
    P, Q = _softmax64(a), _softmax64(b)
    # draft tokens where Q > P strictly, so alpha < 1 and u = 1 rejects; u = 0 accepts
    tok = (Q - P).argmax(-1)
    u = np.zeros((K + 1, K))
    for j in range(K):
        u[j, j] = 1.0
    r = oracle.score_windows(b, a, tok, u, cost_ratio=0.1, want=("accept_prob",))
    assert np.all(r.accept_prob < 1.0)
    assert list(r.accepted_len) == list(range(K)) + [K]
    # the accepted-length formula itself, against "index of the first reject"
    for bits in itertools.product([0, 1], repeat=5):
        first_reject = bits.index(0) if 0 in bits else 5
        assert oracle.accepted_length(bits) == first_reject


def test_acceptance_comparison_is_non_strict_and_alpha_is_the_ratio():
    a = np.log(np.array([[[0.5, 0.25, 0.25]]]))
    b = np.log(np.array([[[0.25, 0.5, 0.25]]]))
    r = _score(a, b, [[1]], [[0.5]], want=("accept_prob",))
    alpha = r.accept_prob[0, 0]                 # P(1)/Q(1) = 0.5
    assert alpha == pytest.approx(0.5, rel=1e-7)
    for u, expect in ((alpha, 1), (np.nextafter(alpha, 1.0), 0), (np.nextafter(alpha, 0.0), 1)):
        r = _score(a, b, [[1]], [[u]])
        assert r.accepted_len[0] == expect
    # target more likely than draft: ratio 2 is clipped to 1, accepted even at u = 1
    r = _score(a, b, [[0]], [[1.0]], want=("accept_prob",))
    assert r.accept_prob[0, 0] == 1.0 and r.accepted_len[0] == 1


# ---- P4: confidence factor --------------------------------------------------------------

def test_confidence_uniform_onehot_and_bounds():
    rng = np.random.default_rng(4)
    V = 1000
    flat = np.full(V, 1.25)
    assert oracle.entropy(flat) == pytest.approx(math.log(V), rel=1e-13)
    assert oracle.confidence(flat) == pytest.approx(0.0, abs=1e-13)
    peaked = np.zeros(V)
    peaked[17] = 50.0
    assert oracle.confidence(peaked) == pytest.approx(1.0, abs=1e-15)
    # uniform target: criticality is zero whatever the drafter says
    b = rng.normal(0, 3, size=(1, 1, V)).astype(np.float32)
    r = oracle.score_windows(b, np.full((1, 1, V), 1.25, np.float32), [[3]], [[0.5]], cost_ratio=0.1)
    assert abs(r.adaw_score[0]) < 1e-12 and r.kl[0, 0] > 0.1
    for _ in range(20):
        a = rng.normal(0, rng.uniform(0.1, 8), size=V)
        assert 0.0 <= oracle.confidence(a) <= 1.0


def test_adaw_score_is_mean_of_confidence_times_kl_over_all_positions():
    rng = np.random.default_rng(5)
    B, K, V = 4, 5, 300
    a = rng.normal(0, 3, size=(B, K, V)).astype(np.float32)
    b = (a + rng.normal(0, 1, size=a.shape)).astype(np.float32)
    tok = rng.integers(0, V, size=(B, K))
    u = np.ones((B, K))                       # reject at once: truncation must not matter
    r = oracle.score_windows(b, a, tok, u, cost_ratio=0.1)
    P = _softmax64(a)
    logP = torch.log_softmax(torch.tensor(a, dtype=torch.float64), -1).numpy()
    logQ = torch.log_softmax(torch.tensor(b, dtype=torch.float64), -1).numpy()
    kl = scipy.special.rel_entr(P, np.exp(logQ)).sum(-1)
    H = scipy.special.entr(P).sum(-1)
    np.testing.assert_allclose(r.kl, kl, rtol=1e-10)
    np.testing.assert_allclose(r.kl, (P * (logP - logQ)).sum(-1), rtol=1e-11)
    np.testing.assert_allclose(r.confidence, 1 - H / math.log(V), rtol=1e-10)
    np.testing.assert_allclose(r.adaw_score, ((1 - H / math.log(V)) * kl).mean(-1), rtol=1e-10)


# ---- P6 / P7: expected acceptance, total variation, Pinsker -------------------------------

def test_expected_accept_equals_one_minus_tv_and_pinsker():
    rng = np.random.default_rng(6)
    for V in (2, 3, 17, 1000):
        for sigma in (0.05, 0.5, 3.0):
            a, b = _rand_pair(rng, V, sigma)
            ea, tv, kl = oracle.expected_accept(a, b), oracle.total_variation(a, b), oracle.kl(a, b)
            assert ea == pytest.approx(1.0 - tv, abs=1e-13)
            assert ea >= 1.0 - math.sqrt(0.5 * kl) - 1e-13
            assert 0.0 <= ea <= 1.0 + 1e-15
            P, Q = _softmax64(a), _softmax64(b)
            assert ea == pytest.approx(np.minimum(P, Q).sum(), rel=1e-12)


@pytest.mark.parametrize("V", [2, 3, 4])
def test_bruteforce_expectation_of_accept_prob_over_drafted_token(V):
    rng = np.random.default_rng(7 + V)
    for _ in range(10):
        a, b = _rand_pair(rng, V, 1.5)
        P, Q = _softmax64(a), _softmax64(b)
        lse_a, lse_b = oracle.logsumexp(a), oracle.logsumexp(b)
        total = 0.0
        for y in range(V):          # enumerate every drafted token
            alpha = oracle.accept_prob(a[y] - lse_a, b[y] - lse_b)
            assert alpha == pytest.approx(min(1.0, P[y] / Q[y]), rel=1e-12)
            total += Q[y] * alpha
        assert total == pytest.approx(oracle.expected_accept(a, b), rel=1e-12)


# ---- P8: brute force over uniforms --------------------------------------------------------

@pytest.mark.parametrize("K", [1, 2, 3])
def test_bruteforce_mean_accepted_length_over_uniform_grid(K):
    rng = np.random.default_rng(20 + K)
    V, N = 4, 40
    a = rng.normal(0, 1.5, size=(1, K, V)).astype(np.float32)
    b = (a + rng.normal(0, 1.5, size=a.shape)).astype(np.float32)
    tok = rng.integers(0, V, size=(1, K))
    P, Q = _softmax64(a)[0], _softmax64(b)[0]
    alpha = np.array([min(1.0, P[t, tok[0, t]] / Q[t, tok[0, t]]) for t in range(K)])
    grid = (np.arange(N) + 0.5) / N
    cells = np.array(list(itertools.product(grid, repeat=K)))          # [N^K, K]
    n = cells.shape[0]
    r = oracle.score_windows(np.repeat(b, n, 0), np.repeat(a, n, 0), np.repeat(tok, n, 0), cells,
                             cost_ratio=0.1)
    expected = sum(np.prod(alpha[:m]) for m in range(1, K + 1))        # E[tau], independent u_t
    assert abs(r.accepted_len.mean() - expected) <= K / N
    first_reject = np.array([next((t for t in range(K) if c[t] > alpha[t]), K) for c in cells])
    assert np.array_equal(r.accepted_len, first_reject)


# ---- P9: softmax statistics against closed forms and library routines --------------------

def test_v2_closed_form_bernoulli():
    for x, y in ((0.3, -1.1), (2.0, 2.0), (-4.0, 3.0)):
        a = np.array([x, 0.0])
        b = np.array([y, 0.0])
        p = 1 / (1 + math.exp(-x))
        q = 1 / (1 + math.exp(-y))
        H = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        KL = p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q))
        assert oracle.entropy(a) == pytest.approx(H, rel=1e-12)
        assert oracle.kl(a, b) == pytest.approx(KL, rel=1e-10, abs=1e-15)
        assert oracle.confidence(a) == pytest.approx(1 - H / math.log(2), rel=1e-11, abs=1e-14)
        assert oracle.expected_accept(a, b) == pytest.approx(min(p, q) + min(1 - p, 1 - q), rel=1e-12)


def test_kl_is_target_to_draft_not_the_reverse():
    rng = np.random.default_rng(9)
    a, b = _rand_pair(rng, 50, 2.0)
    P, Q = _softmax64(a), _softmax64(b)
    fwd, rev = scipy.special.rel_entr(P, Q).sum(), scipy.special.rel_entr(Q, P).sum()
    assert abs(fwd - rev) > 1e-3
    assert oracle.kl(a, b) == pytest.approx(fwd, rel=1e-11)
    r = _score(a.astype(np.float32)[None, None], b.astype(np.float32)[None, None], [[0]], [[0.5]],
               want=("kl", "reverse_kl"))
    P, Q = _softmax64(a.astype(np.float32)), _softmax64(b.astype(np.float32))
    assert r.kl[0, 0] == pytest.approx(scipy.special.rel_entr(P, Q).sum(), rel=1e-11)
    assert r.reverse_kl[0, 0] == pytest.approx(scipy.special.rel_entr(Q, P).sum(), rel=1e-11)


def test_logsumexp_and_argmax_against_library_and_extremes():
    rng = np.random.default_rng(10)
    x = rng.normal(0, 5, size=999)
    assert oracle.logsumexp(x) == pytest.approx(float(scipy.special.logsumexp(x)), rel=1e-14)
    big = np.array([1000.0, 1000.0, -1000.0])
    assert oracle.logsumexp(big) == pytest.approx(1000.0 + math.log(2.0), rel=1e-15)
    assert oracle.argmax(np.array([1.0, 7.0, 7.0, -2.0, 7.0])) == 1     # ties: lowest index
    assert oracle.argmax(x) == int(np.argmax(x))
    # the zero-probability guard: far-away logits contribute nothing, not NaN
    a = np.array([0.0, -2000.0])
    assert oracle.entropy(a) == 0.0
    assert oracle.kl(a, np.array([0.0, 0.0])) == pytest.approx(math.log(2.0), rel=1e-15)


def test_shift_invariance_of_every_output():
    rng = np.random.default_rng(11)
    B, K, V = 3, 4, 128
    a = np.round(rng.normal(0, 3, size=(B, K, V)) * 64) / 64      # exact in fp32 after shifts
    b = a + np.round(rng.normal(0, 1, size=a.shape) * 64) / 64
    tok = rng.integers(0, V, size=(B, K))
    u = rng.random((B, K))
    want = ("kl", "confidence", "accept_prob", "expected_accept", "reverse_kl", "alignment")
    r0 = _score(a, b, tok, u, want=want)
    r1 = _score(a + 8.0, b - 16.0, tok, u, want=want)
    for name in ("r_speedup", "r_proximity", "adaw_score", "delta") + want:
        np.testing.assert_allclose(getattr(r1, name), getattr(r0, name), rtol=1e-10, atol=1e-12)
    assert np.array_equal(r0.accepted_len, r1.accepted_len)


def test_bf16_rows_are_widened_exactly():
    t = (torch.randn(2, 3, 64, generator=torch.Generator().manual_seed(0)) * 5).to(torch.bfloat16)
    row = oracle.widen_row(t[1, 2])
    assert np.array_equal(row, t[1, 2].to(torch.float64).numpy())
    a32 = t.to(torch.float32)
    tok = torch.randint(0, 64, (2, 3)).numpy()
    u = np.full((2, 3), 0.5)
    r16 = oracle.score_windows(t, t.roll(1, -1), tok, u, cost_ratio=0.1)
    r32 = oracle.score_windows(a32, a32.roll(1, -1), tok, u, cost_ratio=0.1)
    assert np.array_equal(r16.kl, r32.kl) and np.array_equal(r16.accepted_len, r32.accepted_len)


# ---- P10 / P11: proximity gap and reward ----------------------------------------------------

def test_proximity_gap_is_lse_free_and_zero_iff_drafted_is_argmax():
    rng = np.random.default_rng(12)
    B, K, V = 5, 4, 90
    a = rng.normal(0, 3, size=(B, K, V)).astype(np.float32)
    b = (a + rng.normal(0, 1, size=a.shape)).astype(np.float32)
    tok = rng.integers(0, V, size=(B, K))
    tok[0] = a[0].argmax(-1)
    r = oracle.score_windows(b, a, tok, np.ones((B, K)), cost_ratio=0.1)
    a64 = a.astype(np.float64)
    gathered = np.take_along_axis(a64, tok[..., None], -1)[..., 0]
    np.testing.assert_allclose(r.delta, (a64.max(-1) - gathered).sum(-1), rtol=1e-12, atol=1e-12)
    assert r.delta[0] == 0.0 and np.all(r.delta[1:] > 0)
    # with a caller-supplied reference the gap is ref - sum_t log P_t(drafted_t)
    logP = torch.log_softmax(torch.tensor(a64), -1).numpy()
    logp_tok = np.take_along_axis(logP, tok[..., None], -1)[..., 0].sum(-1)
    ref = rng.normal(-3, 1, size=B)
    r2 = oracle.score_windows(b, a, tok, np.ones((B, K)), ref, cost_ratio=0.1)
    np.testing.assert_allclose(r2.delta, ref - logp_tok, rtol=1e-12)


def test_proximity_reward_fires_only_at_k0_and_below_eps():
    V, K = 16, 2
    a = np.zeros((4, K, V), np.float32)
    a[:, :, 0] = 4.0                       # target argmax is token 0 everywhere
    a[0, 0, 1] = 4.0 - 0.25                # window 0: gap 0.25 + 0.24 = 0.49 < eps
    a[0, 1, 1] = 4.0 - 0.24
    a[1, 0, 1] = 4.0 - 0.25                # window 1: gap 0.25 + 0.26 = 0.51 > eps
    a[1, 1, 1] = 4.0 - 0.26
    a[2, :, 1] = 4.0 - 0.1                 # window 2: small gap but k >= 1
    a[3, 0, 1] = 4.0 - 0.25                # window 3: gap exactly 0.5 -> strict '<' fails
    a[3, 1, 1] = 4.0 - 0.25
    b = a.copy()
    b[:, :, 1] += 3.0                      # drafter prefers token 1: alpha < 1 there
    tok = np.ones((4, K), np.int64)
    u = np.full((4, K), 0.999)             # reject every drafted token 1 ...
    u[2, 0] = 0.0                          # ... except window 2's first
    r = oracle.score_windows(b, a, tok, u, cost_ratio=0.1, prox_eps=0.5, prox_eta=0.7)
    assert list(r.accepted_len) == [0, 0, 1, 0]
    assert list(r.r_proximity) == [0.7, 0.0, 0.0, 0.0]
    np.testing.assert_allclose(r.delta, [0.49, 0.51, 0.2, 0.5], rtol=0, atol=1e-6)
    assert oracle.proximity_reward(0, 0.1, 0.5, 2.0) == 2.0
    assert oracle.proximity_reward(1, 0.1, 0.5, 2.0) == 0.0


# ---- P12: selection ---------------------------------------------------------------------

def test_select_is_prefix_of_full_stable_sort_with_ties():
    rng = np.random.default_rng(13)
    s = rng.random(500)
    s[[7, 90, 91, 300, 499]] = s.max() + 1.0      # five-way tie at the top
    s[[3, 4]] = s.min() - 1.0
    order = np.lexsort((np.arange(s.size), -s))    # score desc, then index asc
    for M in (1, 3, 5, 6, 250, 500):
        assert np.array_equal(oracle.select_windows(s, M), order[:M])
    assert list(oracle.select_windows(s, 5)) == [7, 90, 91, 300, 499]
    with pytest.raises(ValueError):
        oracle.select_windows(s, 501)
    with pytest.raises(ValueError):
        oracle.select_windows(s, 0)


# ---- by-products: alignment metric and group-relative advantage ---------------------------

def test_alignment_metric_closed_values():
    assert oracle.alignment_metric(-1.0, -1.0) == 0.0
    assert oracle.alignment_metric(-1.0, -2.0) == pytest.approx(math.e - 2.0, rel=1e-15)
    assert oracle.alignment_metric(-2.0, -1.0) == pytest.approx(math.exp(-1.0), rel=1e-15)
    for d in np.linspace(-5, 5, 41):
        assert oracle.alignment_metric(d, 0.0) >= 0.0


def test_group_advantage_is_standardised():
    rng = np.random.default_rng(14)
    r = rng.random(8) * 3
    adv = oracle.group_advantage(r, 1e-6)
    assert abs(adv.sum()) < 1e-9                                   # zero mean
    assert np.array_equal(np.argsort(adv), np.argsort(r))          # order preserved
    np.testing.assert_allclose(adv, (r - r.mean()) / (r.std() + 1e-6), rtol=1e-12)
    assert np.all(oracle.group_advantage(np.full(8, 2.5), 1e-6) == 0.0)


# ---- candidate groups and sequence-mode ADAW (Algorithm 1) -----------------------------------

def test_group_best_is_first_maximum():
    k = [0, 3, 3, 1, 2, 2, 2, 2, 5, 0, 0, 0]
    best, idx = oracle.group_best(k, 4)
    assert list(best) == [3, 2, 5] and list(idx) == [1, 0, 0]
    best, idx = oracle.group_best(k, 1)
    assert list(best) == k and list(idx) == [0] * 12
    with pytest.raises(ValueError):
        oracle.group_best(k, 5)


def test_sequence_scores_match_independent_windows():
    """Scoring T rows once and box-filtering must equal scoring every overlapping window
    on its own (the definition of s_j in Section 4.2)."""
    rng = np.random.default_rng(30)
    N, T, V, K = 2, 9, 200, 4
    a = rng.normal(0, 3, size=(N, T, V)).astype(np.float32)
    b = (a + rng.normal(0, 1, size=a.shape)).astype(np.float32)
    v, s = oracle.adaw_sequence(b, a, K)
    assert v.shape == (N, T) and s.shape == (N, T - K + 1)
    # every overlapping window as an independent [K, V] window of the window-mode scorer
    wa = np.stack([a[n, j:j + K] for n in range(N) for j in range(T - K + 1)])
    wb = np.stack([b[n, j:j + K] for n in range(N) for j in range(T - K + 1)])
    r = oracle.score_windows(wb, wa, np.zeros((wa.shape[0], K), np.int64), np.ones((wa.shape[0], K)),
                             cost_ratio=0.1)
    np.testing.assert_allclose(s.reshape(-1), r.adaw_score, rtol=1e-13)
    np.testing.assert_allclose(v[0, :K], r.confidence[0] * r.kl[0], rtol=1e-13)
    # box filter closed form: s_{j+1} - s_j = (v_{j+K} - v_j) / K
    np.testing.assert_allclose(np.diff(s, axis=1), (v[:, K:] - v[:, :-K]) / K, rtol=1e-9, atol=1e-14)


def test_sample_starts_inverts_the_cumulative_distribution():
    s = np.array([[1.0, 0.0, 3.0, 0.0, 4.0], [0.0, 0.0, 0.0, 0.0, 0.0], [0.0, 2.0, 0.0, 0.0, 0.0]])
    # sequence 0: cumulative shares 0.125, 0.125, 0.5, 0.5, 1.0
    for u, expect in ((0.0, 0), (0.1, 0), (0.125, 0), (0.126, 2), (0.5, 2), (0.51, 4), (0.999, 4)):
        assert oracle.sample_starts(s[:1], [u])[0] == expect
    # all-zero scores: uniform over the W starts; a single nonzero score: always that start
    assert [oracle.sample_starts(s[1:2], [u])[0] for u in (0.0, 0.39, 0.4, 0.99)] == [0, 1, 2, 4]
    assert [oracle.sample_starts(s[2:3], [u])[0] for u in (0.001, 0.5, 0.999)] == [1, 1, 1]
    # frequencies over a fine grid of u approach the normalised weights
    u = (np.arange(8000) + 0.5) / 8000
    picks = oracle.sample_starts(np.repeat(s[:1], u.size, 0), u)
    freq = np.bincount(picks, minlength=5) / u.size
    np.testing.assert_allclose(freq, s[0] / s[0].sum(), atol=2e-4)


def test_curriculum_mixes_adaw_and_uniform_starts_in_the_stated_proportion():
    """Hard-window curriculum (Appendix A.3, Table 5): a fraction rho of the windows is
    ADAW-selected, the rest ordinary.  Over a grid of both draws the start frequencies must be
    rho * s_j / sum(s) + (1 - rho) / W; rho = 1 is plain proportional sampling, rho = 0 plain
    uniform sampling."""
    s = np.array([[1.0, 0.0, 3.0, 0.0, 4.0]])
    W = s.shape[1]
    g = 400
    u_start, u_mix = np.meshgrid((np.arange(g) + 0.5) / g, (np.arange(g) + 0.5) / g)
    u_start, u_mix = u_start.ravel(), u_mix.ravel()
    rows = np.repeat(s, u_start.size, 0)
    for rho in (0.2, 0.4, 0.6):                              # Table 5's schedule
        picks = oracle.sample_starts_curriculum(rows, u_start, u_mix, rho)
        freq = np.bincount(picks, minlength=W) / picks.size
        np.testing.assert_allclose(freq, rho * s[0] / s[0].sum() + (1 - rho) / W, atol=3e-3)
    # a mistake in the direction of the comparison would swap the two shares
    assert abs(freq[1] - 0.4 / W) < 3e-3 and abs(freq[4] - (0.6 * 0.5 + 0.4 / W)) < 3e-3
    only_adaw = oracle.sample_starts_curriculum(rows, u_start, u_mix, 1.0)
    assert np.array_equal(only_adaw, oracle.sample_starts(rows, u_start))
    only_uniform = oracle.sample_starts_curriculum(rows, u_start, u_mix, 0.0)
    assert np.array_equal(only_uniform, np.minimum(np.floor(u_start * W), W - 1).astype(np.int64))
    with pytest.raises(ValueError):
        oracle.sample_starts_curriculum(rows[:1], [0.5], [0.5], 1.5)
