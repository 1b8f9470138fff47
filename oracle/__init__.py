"""ctypes front end of the PPOW window-scoring ORACLE (test infrastructure).

The arithmetic lives in ppow_oracle.c (plain C, double precision, the paper's
definitions written out).  This module only marshals numpy arrays.  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import it; the HIP
product path never does.
"""
import ctypes
import os
from types import SimpleNamespace

import numpy as np

from . import build as _build

F32 = 0
BF16 = 1
REJECTION = 0
GREEDY = 1

_lib = None

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_int32_p = ctypes.POINTER(ctypes.c_int32)
_c_int64_p = ctypes.POINTER(ctypes.c_int64)


class _Outputs(ctypes.Structure):
    _fields_ = [
        ("accepted_len", _c_int32_p),
        ("r_speedup", _c_double_p), ("r_proximity", _c_double_p),
        ("adaw_score", _c_double_p), ("delta", _c_double_p),
        ("kl", _c_double_p), ("confidence", _c_double_p), ("entropy", _c_double_p),
        ("accept_prob", _c_double_p), ("expected_accept", _c_double_p),
        ("reverse_kl", _c_double_p), ("logp_target_tok", _c_double_p),
        ("logp_draft_tok", _c_double_p), ("alignment", _c_double_p),
        ("argmax_target", _c_int64_p),
    ]


def lib():
    """Load (building if needed) the oracle's shared library."""
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        d, i32, i64, vp = ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.ppow_oracle_widen_row.argtypes = [vp, i64, ctypes.c_int, _c_double_p]
        L.ppow_oracle_widen_row.restype = None
        L.ppow_oracle_logsumexp.argtypes = [_c_double_p, i64]
        L.ppow_oracle_logsumexp.restype = d
        L.ppow_oracle_argmax.argtypes = [_c_double_p, i64]
        L.ppow_oracle_argmax.restype = i64
        L.ppow_oracle_entropy.argtypes = [_c_double_p, i64, d]
        L.ppow_oracle_entropy.restype = d
        L.ppow_oracle_kl.argtypes = [_c_double_p, _c_double_p, i64, d, d]
        L.ppow_oracle_kl.restype = d
        L.ppow_oracle_confidence.argtypes = [d, i64]
        L.ppow_oracle_confidence.restype = d
        L.ppow_oracle_expected_accept.argtypes = [_c_double_p, _c_double_p, i64, d, d]
        L.ppow_oracle_expected_accept.restype = d
        L.ppow_oracle_total_variation.argtypes = [_c_double_p, _c_double_p, i64, d, d]
        L.ppow_oracle_total_variation.restype = d
        L.ppow_oracle_accept_prob.argtypes = [d, d]
        L.ppow_oracle_accept_prob.restype = d
        L.ppow_oracle_accepted_length.argtypes = [_c_int32_p, i32]
        L.ppow_oracle_accepted_length.restype = i32
        L.ppow_oracle_speedup_reward.argtypes = [i32, d]
        L.ppow_oracle_speedup_reward.restype = d
        L.ppow_oracle_proximity_reward.argtypes = [i32, d, d, d]
        L.ppow_oracle_proximity_reward.restype = d
        L.ppow_oracle_alignment_metric.argtypes = [d, d]
        L.ppow_oracle_alignment_metric.restype = d
        L.ppow_oracle_group_advantage.argtypes = [_c_double_p, i32, d, _c_double_p]
        L.ppow_oracle_group_advantage.restype = None
        L.ppow_oracle_score_windows.argtypes = [
            vp, vp, _c_int32_p, _c_double_p, _c_double_p, i64, i32, i64, ctypes.c_int,
            d, d, d, ctypes.c_int, ctypes.POINTER(_Outputs), _c_int32_p]
        L.ppow_oracle_score_windows.restype = ctypes.c_int
        L.ppow_oracle_group_best.argtypes = [_c_int32_p, i64, i32, _c_int32_p, _c_int32_p]
        L.ppow_oracle_group_best.restype = ctypes.c_int
        L.ppow_oracle_adaw_sequence.argtypes = [vp, vp, i64, i32, i64, ctypes.c_int, i32,
                                                _c_double_p, _c_double_p]
        L.ppow_oracle_adaw_sequence.restype = ctypes.c_int
        L.ppow_oracle_sample_starts.argtypes = [_c_double_p, i64, i64, _c_double_p, _c_int64_p]
        L.ppow_oracle_sample_starts.restype = ctypes.c_int
        L.ppow_oracle_sample_starts_curriculum.argtypes = [_c_double_p, i64, i64, _c_double_p,
                                                           _c_double_p, d, _c_int64_p]
        L.ppow_oracle_sample_starts_curriculum.restype = ctypes.c_int
        L.ppow_oracle_select_windows.argtypes = [_c_double_p, i64, i64, _c_int64_p]
        L.ppow_oracle_select_windows.restype = ctypes.c_int
        _lib = L
    return _lib


def _dp(a):
    return a.ctypes.data_as(_c_double_p)


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def as_stored(logits):
    """Return (contiguous numpy array of the stored bits, dtype code).

    Accepts numpy float32, numpy uint16 (bfloat16 bit patterns) or a CPU torch
    tensor of dtype float32 / bfloat16.  No value is changed.
    """
    if hasattr(logits, "detach"):  # torch tensor, imported lazily by the caller
        import torch
        t = logits.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16), BF16
        if t.dtype == torch.float32:
            return t.numpy(), F32
        raise TypeError(f"unsupported logits dtype {t.dtype}")
    a = np.ascontiguousarray(logits)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError(f"unsupported logits dtype {a.dtype}")


def widen_row(row):
    a, code = as_stored(row)
    out = np.empty(a.shape[-1], dtype=np.float64)
    lib().ppow_oracle_widen_row(a.ctypes.data, a.shape[-1], code, _dp(out))
    return out


def logsumexp(x):
    x = _f64(x)
    return lib().ppow_oracle_logsumexp(_dp(x), x.size)


def argmax(x):
    x = _f64(x)
    return int(lib().ppow_oracle_argmax(_dp(x), x.size))


def entropy(a):
    a = _f64(a)
    return lib().ppow_oracle_entropy(_dp(a), a.size, logsumexp(a))


def kl(a, b):
    a, b = _f64(a), _f64(b)
    return lib().ppow_oracle_kl(_dp(a), _dp(b), a.size, logsumexp(a), logsumexp(b))


def confidence(a):
    a = _f64(a)
    return lib().ppow_oracle_confidence(entropy(a), a.size)


def expected_accept(a, b):
    a, b = _f64(a), _f64(b)
    return lib().ppow_oracle_expected_accept(_dp(a), _dp(b), a.size, logsumexp(a), logsumexp(b))


def total_variation(a, b):
    a, b = _f64(a), _f64(b)
    return lib().ppow_oracle_total_variation(_dp(a), _dp(b), a.size, logsumexp(a), logsumexp(b))


def accept_prob(logp_target_tok, logp_draft_tok):
    return lib().ppow_oracle_accept_prob(float(logp_target_tok), float(logp_draft_tok))


def accepted_length(accept):
    acc = np.ascontiguousarray(np.asarray(accept, dtype=np.int32))
    return int(lib().ppow_oracle_accepted_length(acc.ctypes.data_as(_c_int32_p), acc.size))


def speedup_reward(k, gamma):
    return lib().ppow_oracle_speedup_reward(int(k), float(gamma))


def proximity_reward(k, delta, eps, eta):
    return lib().ppow_oracle_proximity_reward(int(k), float(delta), float(eps), float(eta))


def alignment_metric(logp_target_tok, logp_draft_tok):
    return lib().ppow_oracle_alignment_metric(float(logp_target_tok), float(logp_draft_tok))


def group_advantage(rewards, delta_stab):
    r = _f64(rewards)
    out = np.empty_like(r)
    lib().ppow_oracle_group_advantage(_dp(r), r.size, float(delta_stab), _dp(out))
    return out


_PER_WINDOW = ("r_speedup", "r_proximity", "adaw_score", "delta")
_PER_POSITION = ("kl", "confidence", "entropy", "accept_prob", "expected_accept", "reverse_kl",
                 "logp_target_tok", "logp_draft_tok", "alignment")


def score_windows(draft_logits, target_logits, draft_tokens, uniforms=None, ref_logprob=None, *,
                  cost_ratio, prox_eps=0.5, prox_eta=1.0, verify=REJECTION,
                  want=("kl", "confidence", "accept_prob")):
    """Score windows with the oracle.  Logits are [B, K, V] stored arrays.

    `want` names the per-position outputs to compute (expected_accept and
    reverse_kl cost one more vocabulary pass each).  Returns a namespace of
    numpy arrays plus `threads`, the number of host threads used.
    """
    b_bits, code_b = as_stored(draft_logits)
    a_bits, code_a = as_stored(target_logits)
    if code_a != code_b or a_bits.shape != b_bits.shape or a_bits.ndim != 3:
        raise ValueError("draft and target logits must share dtype and [B, K, V] shape")
    B, K, V = a_bits.shape
    tok = np.ascontiguousarray(np.asarray(draft_tokens, dtype=np.int32)).reshape(B, K)
    u = None if uniforms is None else _f64(uniforms).reshape(B, K)
    ref = None if ref_logprob is None else _f64(ref_logprob).reshape(B)

    res = SimpleNamespace()
    res.accepted_len = np.zeros(B, dtype=np.int32)
    for name in _PER_WINDOW:
        setattr(res, name, np.zeros(B, dtype=np.float64))
    outs = _Outputs()
    outs.accepted_len = res.accepted_len.ctypes.data_as(_c_int32_p)
    for name in _PER_WINDOW:
        setattr(outs, name, _dp(getattr(res, name)))
    for name in _PER_POSITION:
        if name in want:
            arr = np.zeros((B, K), dtype=np.float64)
            setattr(res, name, arr)
            setattr(outs, name, _dp(arr))
    res.argmax_target = np.zeros((B, K), dtype=np.int64)
    outs.argmax_target = res.argmax_target.ctypes.data_as(_c_int64_p)

    threads = ctypes.c_int32(0)
    rc = lib().ppow_oracle_score_windows(
        b_bits.ctypes.data, a_bits.ctypes.data, tok.ctypes.data_as(_c_int32_p),
        None if u is None else _dp(u), None if ref is None else _dp(ref),
        B, K, V, code_a, float(cost_ratio), float(prox_eps), float(prox_eta), int(verify),
        ctypes.byref(outs), ctypes.byref(threads))
    if rc != 0:
        raise ValueError("ppow_oracle_score_windows rejected its arguments")
    res.threads = int(threads.value)
    return res


def group_best(accepted_len, group):
    """(best accepted length, index of the first window attaining it) per group of windows."""
    k = np.ascontiguousarray(np.asarray(accepted_len, dtype=np.int32)).reshape(-1)
    if group < 1 or k.size % group:
        raise ValueError("group must divide the number of windows")
    best = np.empty(k.size // group, dtype=np.int32)
    idx = np.empty(k.size // group, dtype=np.int32)
    rc = lib().ppow_oracle_group_best(k.ctypes.data_as(_c_int32_p), k.size, int(group),
                                      best.ctypes.data_as(_c_int32_p), idx.ctypes.data_as(_c_int32_p))
    if rc != 0:
        raise ValueError("ppow_oracle_group_best rejected its arguments")
    return best, idx


def adaw_sequence(draft_logits, target_logits, K):
    """Sequence-mode ADAW: (criticality [N, T], window_score [N, T-K+1]) for [N, T, V] logits."""
    b_bits, code_b = as_stored(draft_logits)
    a_bits, code_a = as_stored(target_logits)
    if code_a != code_b or a_bits.shape != b_bits.shape or a_bits.ndim != 3:
        raise ValueError("draft and target logits must share dtype and [N, T, V] shape")
    N, T, V = a_bits.shape
    v = np.zeros((N, T), dtype=np.float64)
    s = np.zeros((N, T - K + 1), dtype=np.float64)
    rc = lib().ppow_oracle_adaw_sequence(b_bits.ctypes.data, a_bits.ctypes.data, N, T, V, code_a,
                                         int(K), _dp(v), _dp(s))
    if rc != 0:
        raise ValueError("ppow_oracle_adaw_sequence rejected its arguments")
    return v, s


def sample_starts(score, uniforms):
    """One window start per sequence, drawn with probability proportional to the scores."""
    s = _f64(score)
    if s.ndim != 2:
        raise ValueError("score must be [N, W]")
    u = _f64(uniforms).reshape(-1)
    out = np.empty(s.shape[0], dtype=np.int64)
    rc = lib().ppow_oracle_sample_starts(_dp(s), s.shape[0], s.shape[1], _dp(u),
                                         out.ctypes.data_as(_c_int64_p))
    if rc != 0:
        raise ValueError("ppow_oracle_sample_starts rejected its arguments")
    return out


def sample_starts_curriculum(score, uniforms, mix_uniforms, adaw_fraction):
    """Window starts under the hard-window curriculum: ADAW-selected (proportional to the
    scores) where mix_uniforms < adaw_fraction, uniformly random otherwise."""
    s = _f64(score)
    if s.ndim != 2:
        raise ValueError("score must be [N, W]")
    u = _f64(uniforms).reshape(-1)
    m = _f64(mix_uniforms).reshape(-1)
    out = np.empty(s.shape[0], dtype=np.int64)
    rc = lib().ppow_oracle_sample_starts_curriculum(_dp(s), s.shape[0], s.shape[1], _dp(u), _dp(m),
                                                    float(adaw_fraction),
                                                    out.ctypes.data_as(_c_int64_p))
    if rc != 0:
        raise ValueError("ppow_oracle_sample_starts_curriculum rejected its arguments")
    return out


def select_windows(score, M):
    s = _f64(score).reshape(-1)
    idx = np.empty(int(M), dtype=np.int64)
    rc = lib().ppow_oracle_select_windows(_dp(s), s.size, int(M), idx.ctypes.data_as(_c_int64_p))
    if rc != 0:
        raise ValueError("ppow_oracle_select_windows rejected its arguments")
    return idx


def set_threads(n):
    """Limit the OpenMP team of later calls (0 or None: leave the default)."""
    if n:
        os.environ["OMP_NUM_THREADS"] = str(int(n))
        try:
            ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        except OSError:
            pass
