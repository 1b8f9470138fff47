"""ctypes binding of libppow: argument marshalling only.

Every step of the scoring path runs in the HIP kernels of libppow.so; torch is
used for device memory and the current stream.  There is no CPU fallback: if the
library is missing or no GPU is visible the calls raise.
"""
import atexit
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PPOW_LIBRARY selects another build of the same library (e.g. a tuning variant)
LIBRARY = os.environ.get("PPOW_LIBRARY") or os.path.join(_HERE, "libppow.so")

PPOW_OK = 0
PPOW_ERR_INVALID_ARG = 1
PPOW_ERR_UNSUPPORTED = 2
PPOW_ERR_WORKSPACE = 3
PPOW_ERR_DEVICE = 4

PPOW_F32 = 0
PPOW_BF16 = 1
PPOW_VERIFY_REJECTION = 0
PPOW_VERIFY_GREEDY = 1
PPOW_FLAG_EXPECTED_ACCEPT = 1
PPOW_FLAG_POLICY_TERMS = 2
PPOW_MAX_K = 64
PPOW_STATIC_MAX_ROWS = 131072

_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)


class PpowParams(ctypes.Structure):
    _fields_ = [("cost_ratio", ctypes.c_float), ("prox_eps", ctypes.c_float),
                ("prox_eta", ctypes.c_float), ("verify", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("rollout_group", ctypes.c_int32),
                ("adv_delta", ctypes.c_float)]


class PpowOutputs(ctypes.Structure):
    _fields_ = [("accepted_len", ctypes.c_void_p), ("r_speedup", ctypes.c_void_p),
                ("r_proximity", ctypes.c_void_p), ("adaw_score", ctypes.c_void_p),
                ("delta", ctypes.c_void_p), ("kl", ctypes.c_void_p),
                ("confidence", ctypes.c_void_p), ("accept_prob", ctypes.c_void_p),
                ("expected_accept", ctypes.c_void_p), ("logp_target_tok", ctypes.c_void_p),
                ("logp_draft_tok", ctypes.c_void_p), ("reverse_kl", ctypes.c_void_p),
                ("alignment", ctypes.c_void_p), ("reverse_kl_mean", ctypes.c_void_p),
                ("alignment_mean", ctypes.c_void_p), ("advantage", ctypes.c_void_p),
                ("group_best_len", ctypes.c_void_p), ("group_best_index", ctypes.c_void_p)]


class PpowError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libppow status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Load libppow.so (built in-tree by paper_2605_14978_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            raise ImportError(f"{LIBRARY} is not built: run `python -m paper_2605_14978_amd.build`")
        L = ctypes.CDLL(LIBRARY)
        vp, i64, i32, u32, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32,
                                 ctypes.c_size_t)
        L.ppow_score_workspace_bytes.argtypes = [i64, i32, i64, i32, u32]
        L.ppow_score_workspace_bytes.restype = sz
        L.ppow_score_windows.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32,
                                         ctypes.POINTER(PpowParams), ctypes.POINTER(PpowOutputs),
                                         vp, sz, vp]
        L.ppow_score_windows.restype = ctypes.c_int
        L.ppow_score_windows_static.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32,
                                                ctypes.POINTER(PpowParams),
                                                ctypes.POINTER(PpowOutputs), vp]
        L.ppow_score_windows_static.restype = ctypes.c_int
        L.ppow_release.argtypes = []
        L.ppow_release.restype = ctypes.c_int
        L.ppow_debug_cluster_wait_limit.argtypes = [u32]
        L.ppow_debug_cluster_wait_limit.restype = None
        L.ppow_adaw_sequence_workspace_bytes.argtypes = [i64, i32, i64, i32]
        L.ppow_adaw_sequence_workspace_bytes.restype = sz
        L.ppow_adaw_sequence.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, ctypes.c_float, vp,
                                         vp, vp, vp, vp, sz, vp]
        L.ppow_adaw_sequence.restype = ctypes.c_int
        L.ppow_select_workspace_bytes.argtypes = [i64, i32]
        L.ppow_select_workspace_bytes.restype = sz
        L.ppow_select_windows.argtypes = [vp, i64, i32, vp, vp, vp, sz, vp]
        L.ppow_select_windows.restype = ctypes.c_int
        L.ppow_last_error.argtypes = []
        L.ppow_last_error.restype = ctypes.c_char_p
        L.ppow_last_row_kernel.argtypes = []
        L.ppow_last_row_kernel.restype = ctypes.c_char_p
        L.ppow_version.argtypes = []
        L.ppow_version.restype = ctypes.c_char_p
        _lib = L
        # the event the library keeps per device goes before the HIP runtime is torn down
        atexit.register(L.ppow_release)
    return _lib


def last_row_kernel():
    """Name of the streaming kernel the last scoring call of this thread launched."""
    return lib().ppow_last_row_kernel().decode()


def _check(status):
    if status != PPOW_OK:
        raise PpowError(status, lib().ppow_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return PPOW_F32
    if t.dtype == torch.bfloat16:
        return PPOW_BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


OPTIONAL_OUTPUTS = ("delta", "kl", "confidence", "accept_prob", "expected_accept",
                    "logp_target_tok", "logp_draft_tok", "reverse_kl", "alignment",
                    "reverse_kl_mean", "alignment_mean", "advantage")
PER_WINDOW_OPTIONAL = ("delta", "reverse_kl_mean", "alignment_mean", "advantage")
PER_GROUP_OPTIONAL = ("group_best_len", "group_best_index")      # int32 [B / rollout_group]


class ScoreBuffers:
    """Device outputs and workspace of ppow_score_windows, allocated once and reused."""

    def __init__(self, B, K, V, dtype_code, device, optional=(), flags=0, rollout_group=0,
                 workspace=True):
        self.B, self.K = B, K
        self.rollout_group = rollout_group
        dev = torch.device(device)
        self.accepted_len = torch.empty(B, dtype=torch.int32, device=dev)
        self.r_speedup = torch.empty(B, dtype=torch.float32, device=dev)
        self.r_proximity = torch.empty(B, dtype=torch.float32, device=dev)
        self.adaw_score = torch.empty(B, dtype=torch.float32, device=dev)
        for name in OPTIONAL_OUTPUTS:
            t = None
            if name in optional:
                n = B if name in PER_WINDOW_OPTIONAL else B * K
                t = torch.empty(n, dtype=torch.float32, device=dev)
                if name not in PER_WINDOW_OPTIONAL:
                    t = t.view(B, K)
            setattr(self, name, t)
        for name in PER_GROUP_OPTIONAL:
            t = None
            if name in optional:
                if rollout_group < 1 or B % rollout_group:
                    raise ValueError("group outputs need rollout_group >= 1 dividing B")
                t = torch.empty(B // rollout_group, dtype=torch.int32, device=dev)
            setattr(self, name, t)
        self.workspace = None           # ppow_score_windows_static brings its own scratch
        if workspace:
            nbytes = lib().ppow_score_workspace_bytes(B, K, V, dtype_code, flags)
            if nbytes == 0:
                raise PpowError(PPOW_ERR_INVALID_ARG, "sizes rejected by ppow_score_workspace_bytes")
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def window_slice(self, w0, w1):
        """A view of these buffers covering windows [w0, w1) (for chunked scoring)."""
        view = object.__new__(ScoreBuffers)
        view.B, view.K = w1 - w0, self.K
        view.rollout_group = self.rollout_group
        for name in ("accepted_len", "r_speedup", "r_proximity", "adaw_score") + OPTIONAL_OUTPUTS:
            t = getattr(self, name)
            setattr(view, name, None if t is None else t[w0:w1])
        for name in PER_GROUP_OPTIONAL:
            t = getattr(self, name)
            g = max(self.rollout_group, 1)
            setattr(view, name, None if t is None else t[w0 // g:w1 // g])
        view.workspace = self.workspace     # shared: calls on one stream run one after another
        return view

    def status(self):
        """First word of the workspace: 0 unless the cluster kernel's bounded wait expired
        (the windows of that call then carry accepted_len = -3)."""
        if self.workspace is None:
            return int((self.accepted_len == -3).any().item())
        return int(self.workspace[:4].view(torch.int32).item())

    def as_struct(self):
        o = PpowOutputs()
        for name, _ in PpowOutputs._fields_:
            t = getattr(self, name)
            setattr(o, name, None if t is None else t.data_ptr())
        return o


def _marshal_score(draft_logits, target_logits, draft_tokens, uniforms, ref_logprob):
    """Shape / dtype checks shared by the two scoring entry points; returns (B, K, V, code)."""
    if not target_logits.is_cuda:
        raise RuntimeError("libppow scores device tensors only; there is no CPU path")
    B, K, V = target_logits.shape
    if draft_logits.shape != target_logits.shape or draft_logits.dtype != target_logits.dtype:
        raise ValueError("draft and target logits must share shape and dtype")
    for t in (draft_logits, target_logits, draft_tokens, uniforms, ref_logprob):
        if t is not None and not t.is_contiguous():
            raise ValueError("all inputs must be contiguous")
    if draft_tokens.dtype != torch.int32 or draft_tokens.numel() != B * K:
        raise ValueError("draft_tokens must be int32 [B, K]")
    if uniforms is not None and (uniforms.dtype != torch.float32 or uniforms.numel() != B * K):
        raise ValueError("uniforms must be float32 [B, K]")
    if ref_logprob is not None and (ref_logprob.dtype != torch.float32 or ref_logprob.numel() != B):
        raise ValueError("ref_logprob must be float32 [B]")
    return B, K, V, _dtype_code(target_logits)


def ppow_score_windows(draft_logits, target_logits, draft_tokens, uniforms=None, ref_logprob=None,
                       *, cost_ratio, prox_eps=0.5, prox_eta=1.0, verify=PPOW_VERIFY_REJECTION,
                       flags=0, rollout_group=0, adv_delta=1e-6, optional=(), buffers=None,
                       stream=None):
    """Score B windows on the GPU; returns the ScoreBuffers holding the device outputs.

    Tensors are CUDA tensors: logits [B, K, V] contiguous float32 / bfloat16,
    draft_tokens [B, K] int32, uniforms [B, K] float32 (None for greedy),
    ref_logprob [B] float32 or None.  The call is asynchronous on `stream`
    (default: torch's current stream).
    """
    B, K, V, code = _marshal_score(draft_logits, target_logits, draft_tokens, uniforms, ref_logprob)
    if buffers is None:
        buffers = ScoreBuffers(B, K, V, code, target_logits.device, optional, flags, rollout_group)
    if buffers.workspace is None:
        raise ValueError("these buffers have no workspace: use ppow_score_windows_static")
    params = PpowParams(float(cost_ratio), float(prox_eps), float(prox_eta), int(verify), int(flags),
                        int(rollout_group), float(adv_delta))
    outs = buffers.as_struct()
    _check(lib().ppow_score_windows(
        _ptr(draft_logits), _ptr(target_logits), _ptr(draft_tokens), _ptr(uniforms),
        _ptr(ref_logprob), B, K, V, code, ctypes.byref(params), ctypes.byref(outs),
        _ptr(buffers.workspace), buffers.workspace.numel(), _stream_handle(stream)))
    return buffers


def ppow_score_windows_static(draft_logits, target_logits, draft_tokens, uniforms=None,
                              ref_logprob=None, *, cost_ratio, prox_eps=0.5, prox_eta=1.0,
                              verify=PPOW_VERIFY_REJECTION, flags=0, rollout_group=0,
                              adv_delta=1e-6, buffers, stream=None):
    """ppow_score_windows without a workspace: the library's built-in scratch is used, nothing
    is allocated by the call (`buffers` are the caller's preallocated outputs, e.g.
    ScoreBuffers(..., workspace=False)).  B*K <= PPOW_STATIC_MAX_ROWS; calls that overlap on
    one GPU race."""
    B, K, V, code = _marshal_score(draft_logits, target_logits, draft_tokens, uniforms, ref_logprob)
    params = PpowParams(float(cost_ratio), float(prox_eps), float(prox_eta), int(verify), int(flags),
                        int(rollout_group), float(adv_delta))
    outs = buffers.as_struct()
    _check(lib().ppow_score_windows_static(
        _ptr(draft_logits), _ptr(target_logits), _ptr(draft_tokens), _ptr(uniforms),
        _ptr(ref_logprob), B, K, V, code, ctypes.byref(params), ctypes.byref(outs),
        _stream_handle(stream)))
    return buffers


class SequenceBuffers:
    """Device outputs and workspace of ppow_adaw_sequence."""

    def __init__(self, N, T, V, K, dtype_code, device, sample=True):
        dev = torch.device(device)
        self.N, self.T, self.K = N, T, K
        self.criticality = torch.empty(N, T, dtype=torch.float32, device=dev)
        self.window_score = torch.empty(N, T - K + 1, dtype=torch.float32, device=dev)
        self.sampled_start = torch.empty(N, dtype=torch.int32, device=dev) if sample else None
        nbytes = lib().ppow_adaw_sequence_workspace_bytes(N, T, V, dtype_code)
        if nbytes == 0:
            raise PpowError(PPOW_ERR_INVALID_ARG, "sizes rejected by ppow_adaw_sequence_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)


def ppow_adaw_sequence(draft_logits, target_logits, K, uniforms=None, *, adaw_fraction=1.0,
                       mix_uniforms=None, buffers=None, stream=None):
    """Sequence-mode ADAW on [N, T, V] teacher-forced logits; returns the SequenceBuffers.

    With `uniforms` ([N] float32) one window start per sequence is drawn: in proportion to
    the window scores where mix_uniforms[n] < adaw_fraction (always, for adaw_fraction = 1),
    uniformly otherwise (hard-window curriculum).  Asynchronous on `stream` (default: torch's
    current stream).
    """
    if not target_logits.is_cuda:
        raise RuntimeError("libppow scores device tensors only; there is no CPU path")
    N, T, V = target_logits.shape
    if draft_logits.shape != target_logits.shape or draft_logits.dtype != target_logits.dtype:
        raise ValueError("draft and target logits must share shape and dtype")
    if not (draft_logits.is_contiguous() and target_logits.is_contiguous()):
        raise ValueError("logits must be contiguous")
    for name, t in (("uniforms", uniforms), ("mix_uniforms", mix_uniforms)):
        if t is not None and (t.dtype != torch.float32 or t.numel() != N or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous float32 [N]")
    code = _dtype_code(target_logits)
    if buffers is None:
        buffers = SequenceBuffers(N, T, V, K, code, target_logits.device, sample=uniforms is not None)
    _check(lib().ppow_adaw_sequence(
        _ptr(draft_logits), _ptr(target_logits), N, T, V, code, int(K), _ptr(uniforms),
        float(adaw_fraction), _ptr(mix_uniforms),
        _ptr(buffers.criticality), _ptr(buffers.window_score),
        _ptr(buffers.sampled_start) if uniforms is not None else None,
        _ptr(buffers.workspace), buffers.workspace.numel(), _stream_handle(stream)))
    return buffers


class SelectBuffers:
    """Device outputs and workspace of ppow_select_windows."""

    def __init__(self, B, M, device):
        dev = torch.device(device)
        self.indices = torch.empty(M, dtype=torch.int32, device=dev)
        self.scores = torch.empty(M, dtype=torch.float32, device=dev)
        nbytes = lib().ppow_select_workspace_bytes(B, M)
        if nbytes == 0:
            raise PpowError(PPOW_ERR_INVALID_ARG, "sizes rejected by ppow_select_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)


def ppow_select_windows(adaw_score, M, *, buffers=None, stream=None):
    """Indices (int32 [M]) of the M largest scores, score descending then index ascending."""
    if not adaw_score.is_cuda:
        raise RuntimeError("libppow selects on device tensors only; there is no CPU path")
    if adaw_score.dtype != torch.float32 or not adaw_score.is_contiguous():
        raise ValueError("adaw_score must be a contiguous float32 tensor")
    B = adaw_score.numel()
    if buffers is None:
        buffers = SelectBuffers(B, M, adaw_score.device)
    _check(lib().ppow_select_windows(
        _ptr(adaw_score), B, int(M), _ptr(buffers.indices), _ptr(buffers.scores),
        _ptr(buffers.workspace), buffers.workspace.numel(), _stream_handle(stream)))
    return buffers
