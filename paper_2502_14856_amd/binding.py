"""ctypes marshalling for libfrspec.so.  Names and argument order follow include/frspec.h.

Tensors are torch CUDA (ROCm) tensors: bf16 data may be passed as ``torch.bfloat16``
or as its bit patterns (``torch.int16`` / ``torch.uint16``).  Work is enqueued on
torch's current stream unless ``stream`` (a raw hipStream_t integer) is given.
"""

from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfrspec.so")

FR_K_MAX = 64


class FrSpecError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {fr_strerror(status)} (status {status})")


class Tuning(ctypes.Structure):
    """Mirror of ``fr_tuning`` (include/frspec_dev.h); zero fields mean library default."""
    _fields_ = [("path", ctypes.c_int32), ("two_launch", ctypes.c_int32),
                ("variant", ctypes.c_int32), ("ksplit", ctypes.c_int32),
                ("grid", ctypes.c_int32), ("stream_only", ctypes.c_int32),
                ("skew", ctypes.c_int32), ("no_mailbox", ctypes.c_int32),
                ("spin_limit", ctypes.c_int32), ("chunked_only", ctypes.c_int32),
                ("trace", ctypes.c_void_p)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  Fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2502_14856_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        L.fr_strerror.argtypes = [ctypes.c_int]
        L.fr_strerror.restype = ctypes.c_char_p
        L.fr_version.argtypes = []
        L.fr_version.restype = ctypes.c_int
        L.fr_build_subset.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, vp]
        L.fr_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.fr_workspace_bytes.restype = sz
        L.fr_workspace_init.argtypes = [vp, sz, vp]
        L.fr_workspace_check.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_int32), vp]
        L.fr_draft_topk.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp, sz, vp]
        L.fr_draft_topk_tuned.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp, sz, vp,
                                          ctypes.POINTER(Tuning)]
        L.fr_full_topk.argtypes = [vp, i64, i64, vp, i64, i32, vp, vp, vp, sz, vp]
        L.fr_draft_logits.argtypes = [vp, i64, i64, vp, i64, vp, vp]
        L.fr_draft_topk_multi.argtypes = [ctypes.POINTER(ctypes.c_void_p), i32, i64, i64, vp, vp, i64, i32, vp, vp,
                                          vp, sz, vp]
        L.fr_count_tokens.argtypes = [vp, i64, i64, vp, vp, vp]
        L.fr_rank_tokens.argtypes = [vp, i64, vp, vp]
        L.fr_tiled_bytes.argtypes = [i64, i64]
        L.fr_tiled_bytes.restype = sz
        L.fr_build_subset_tiled.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, vp]
        L.fr_draft_topk_tiled.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp, sz, vp]
        L.fr_draft_topk_tiled_tuned.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp, sz, vp,
                                                ctypes.POINTER(Tuning)]
        L.fr_init.argtypes = []
        L.fr_draft_topk_static.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp]
        L.fr_draft_step.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, vp,
                                    vp, sz, vp]
        L.fr_beam_expand.argtypes = [vp, vp, i64, i32, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp]
        L.fr_tree_select.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp]
        L.fr_calib_copy.argtypes = [vp, vp, sz, vp]
        L.fr_calib_read.argtypes = [vp, sz, vp, vp]
        for name in ("fr_build_subset", "fr_workspace_init", "fr_workspace_check", "fr_draft_topk", "fr_draft_topk_tuned",
                     "fr_full_topk", "fr_draft_logits", "fr_beam_expand", "fr_tree_select", "fr_draft_step", "fr_draft_topk_multi", "fr_count_tokens", "fr_rank_tokens", "fr_build_subset_tiled",
                     "fr_draft_topk_tiled", "fr_draft_topk_tiled_tuned", "fr_init", "fr_draft_topk_static", "fr_calib_copy",
                     "fr_calib_read"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def fr_strerror(status: int) -> str:
    return lib().fr_strerror(int(status)).decode()


def fr_version() -> int:
    return int(lib().fr_version())


def fr_init() -> None:
    """One-time set-up of the current device (see frspec.h); needed before a stream capture."""
    _check(lib().fr_init(), "fr_init")


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _is_bf16_like(t):
    return t.dtype in (torch.bfloat16, torch.int16, torch.uint16)


def _check(status, what):
    if status != 0:
        raise FrSpecError(status, what)


def _bf16_matrix(t, name):
    if not (t.is_cuda and t.dim() == 2 and t.is_contiguous() and _is_bf16_like(t)):
        raise ValueError(f"{name} must be a contiguous 2-D CUDA tensor of bf16 (or its 16-bit patterns)")
    return t


def fr_workspace_bytes(M: int, d: int, V_rows: int, k: int) -> int:
    return int(lib().fr_workspace_bytes(M, d, V_rows, k))


def fr_workspace_init(workspace, stream=None) -> None:
    _check(lib().fr_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)), "fr_workspace_init")


def fr_workspace_check(workspace, stream=None) -> bool:
    """True if a bounded in-kernel wait ever ran out on this workspace (synchronises)."""
    flag = ctypes.c_int32(0)
    _check(lib().fr_workspace_check(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                    ctypes.byref(flag), _stream(stream)), "fr_workspace_check")
    return bool(flag.value)


def new_workspace(M: int, d: int, V_rows: int, k: int, device="cuda", stream=None):
    """Allocates (torch) and prepares a workspace large enough for the given problem."""
    n = fr_workspace_bytes(M, d, V_rows, k)
    if n == 0:
        raise ValueError("invalid problem size for a workspace")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    fr_workspace_init(ws, stream)
    return ws


def fr_build_subset(W_full, freq_ranked_ids, V_sub: int, W_sub=None, idx_map=None,
                    dev_error_flag=None, stream=None):
    """Eq. 3.  Returns (W_sub, idx_map); outputs are allocated if not supplied."""
    _bf16_matrix(W_full, "W_full")
    V, d = W_full.shape
    if not (freq_ranked_ids.is_cuda and freq_ranked_ids.dtype == torch.int32
            and freq_ranked_ids.is_contiguous() and freq_ranked_ids.numel() >= V_sub):
        raise ValueError("freq_ranked_ids must be a contiguous CUDA int32 tensor with >= V_sub entries")
    if W_sub is None:
        W_sub = torch.empty((V_sub, d), dtype=W_full.dtype, device=W_full.device)
    if idx_map is None:
        idx_map = torch.empty(V_sub, dtype=torch.int32, device=W_full.device)
    _check(lib().fr_build_subset(_ptr(W_full), V, d, _ptr(freq_ranked_ids), V_sub, _ptr(W_sub),
                                 _ptr(idx_map), _ptr(dev_error_flag), _stream(stream)),
           "fr_build_subset")
    return W_sub, idx_map


def _head_outputs(M, k, device, token_ids, logp):
    if token_ids is None:
        token_ids = torch.empty((M, k), dtype=torch.int32, device=device)
    if logp is None:
        logp = torch.empty((M, k), dtype=torch.float32, device=device)
    return token_ids, logp


def fr_draft_topk(H, W_sub, idx_map, k: int, workspace, token_ids=None, logp=None, stream=None,
                  tuning: Tuning | None = None):
    """Eq. 4 + per-row top-k + id remap.  Returns (token_ids int32 [M,k], logp fp32 [M,k])."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W_sub, "W_sub")
    M, d = H.shape
    V_sub = W_sub.shape[0]
    if W_sub.shape[1] != d:
        raise ValueError("H and W_sub disagree on d")
    if idx_map is not None and not (idx_map.is_cuda and idx_map.dtype == torch.int32
                                    and idx_map.is_contiguous() and idx_map.numel() >= V_sub):
        raise ValueError("idx_map must be a contiguous CUDA int32 tensor with >= V_sub entries")
    token_ids, logp = _head_outputs(M, k, H.device, token_ids, logp)
    ws_bytes = workspace.numel() * workspace.element_size()
    if tuning is None:
        st = lib().fr_draft_topk(_ptr(H), M, d, _ptr(W_sub), _ptr(idx_map), V_sub, k,
                                 _ptr(token_ids), _ptr(logp), _ptr(workspace), ws_bytes,
                                 _stream(stream))
    else:
        st = lib().fr_draft_topk_tuned(_ptr(H), M, d, _ptr(W_sub), _ptr(idx_map), V_sub, k,
                                       _ptr(token_ids), _ptr(logp), _ptr(workspace), ws_bytes,
                                       _stream(stream), ctypes.byref(tuning))
    _check(st, "fr_draft_topk")
    return token_ids, logp


def bind_draft_topk(H, W_sub, idx_map, k: int, workspace, token_ids, logp, stream=None):
    """fr_draft_topk with its arguments checked and marshalled once: returns a function of no
    arguments that makes the C call on the same buffers each time it is called (a drafting loop
    repeats one call; the per-call checks of fr_draft_topk cost more host time than the launch).
    The stream is fixed when the call is bound.  Returns the status-checking callable."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W_sub, "W_sub")
    M, d = H.shape
    V_sub = W_sub.shape[0]
    if W_sub.shape[1] != d:
        raise ValueError("H and W_sub disagree on d")
    if idx_map is not None and not (idx_map.is_cuda and idx_map.dtype == torch.int32
                                    and idx_map.is_contiguous() and idx_map.numel() >= V_sub):
        raise ValueError("idx_map must be a contiguous CUDA int32 tensor with >= V_sub entries")
    if tuple(token_ids.shape) != (M, k) or tuple(logp.shape) != (M, k) or token_ids.dtype != torch.int32 \
            or logp.dtype != torch.float32 or not (token_ids.is_contiguous() and logp.is_contiguous()):
        raise ValueError("token_ids / logp must be contiguous int32 / float32 [M, k]")
    fn = lib().fr_draft_topk
    args = (_ptr(H), M, d, _ptr(W_sub), _ptr(idx_map), V_sub, k, _ptr(token_ids), _ptr(logp), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream))
    keep = (H, W_sub, idx_map, workspace, token_ids, logp)     # the buffers live as long as the bound call

    def call(_keep=keep):
        st = fn(*args)
        if st != 0:
            raise FrSpecError(st, "fr_draft_topk")
    return call


def fr_draft_topk_static(H, W_sub, idx_map, k: int, token_ids, logp, stream=None):
    """fr_draft_topk on the library's static scratch (M <= 16, k <= 16).  Allocates nothing:
    the outputs are the caller's."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W_sub, "W_sub")
    M, d = H.shape
    V_sub = W_sub.shape[0]
    if W_sub.shape[1] != d:
        raise ValueError("H and W_sub disagree on d")
    if tuple(token_ids.shape) != (M, k) or tuple(logp.shape) != (M, k) or token_ids.dtype != torch.int32 \
            or logp.dtype != torch.float32 or not (token_ids.is_contiguous() and logp.is_contiguous()):
        raise ValueError("token_ids / logp must be contiguous int32 / float32 [M, k]")
    _check(lib().fr_draft_topk_static(_ptr(H), M, d, _ptr(W_sub), _ptr(idx_map), V_sub, k, _ptr(token_ids),
                                      _ptr(logp), _stream(stream)), "fr_draft_topk_static")
    return token_ids, logp


def fr_full_topk(H, W_full, k: int, workspace, token_ids=None, logp=None, stream=None):
    """Eq. 2 with the same candidate selection.  Returns (token_ids, logp)."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W_full, "W_full")
    M, d = H.shape
    V = W_full.shape[0]
    if W_full.shape[1] != d:
        raise ValueError("H and W_full disagree on d")
    token_ids, logp = _head_outputs(M, k, H.device, token_ids, logp)
    _check(lib().fr_full_topk(_ptr(H), M, d, _ptr(W_full), V, k, _ptr(token_ids), _ptr(logp),
                              _ptr(workspace), workspace.numel() * workspace.element_size(),
                              _stream(stream)), "fr_full_topk")
    return token_ids, logp


def fr_draft_logits(H, W, z_out=None, stream=None):
    """Verification aid: the logits of Eq. 4 as fp32 [M, V_rows]."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W, "W")
    M, d = H.shape
    V_rows = W.shape[0]
    if z_out is None:
        z_out = torch.empty((M, V_rows), dtype=torch.float32, device=H.device)
    _check(lib().fr_draft_logits(_ptr(H), M, d, _ptr(W), V_rows, _ptr(z_out), _stream(stream)),
           "fr_draft_logits")
    return z_out


def fr_draft_topk_multi(H_blocks, W_sub, idx_map, k: int, workspace, token_ids=None, logp=None, stream=None):
    """fr_draft_topk over several equally shaped blocks of hidden states (a list of [rows, d]
    tensors) against one W_sub, in one launch when they have at most 16 rows together."""
    for h in H_blocks:
        _bf16_matrix(h, "H block")
    rows, d = H_blocks[0].shape
    if any(h.shape != (rows, d) for h in H_blocks):
        raise ValueError("all blocks of hidden states must have the same shape")
    _bf16_matrix(W_sub, "W_sub")
    M = rows * len(H_blocks)
    if token_ids is None:
        token_ids = torch.empty((M, k), dtype=torch.int32, device=W_sub.device)
    if logp is None:
        logp = torch.empty((M, k), dtype=torch.float32, device=W_sub.device)
    ptrs = (ctypes.c_void_p * len(H_blocks))(*[h.data_ptr() for h in H_blocks])
    _check(lib().fr_draft_topk_multi(ptrs, len(H_blocks), rows, d, _ptr(W_sub), _ptr(idx_map), W_sub.shape[0], k,
                                     _ptr(token_ids), _ptr(logp), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)),
           "fr_draft_topk_multi")
    return token_ids, logp


def fr_count_tokens(tokens, V: int, counts=None, dev_error_flag=None, stream=None):
    """Adds the occurrences of every id of the int32 stream to counts (int64 [V], created zeroed
    if not given).  Section 3.2: corpus-level token statistics."""
    _dev(tokens, torch.int32, "tokens")
    if counts is None:
        counts = torch.zeros(V, dtype=torch.int64, device=tokens.device)
    _dev(counts, torch.int64, "counts")
    if counts.numel() < V:
        raise ValueError("counts must hold V entries")
    _check(lib().fr_count_tokens(_ptr(tokens), tokens.numel(), V, _ptr(counts), _ptr(dev_error_flag),
                                 _stream(stream)), "fr_count_tokens")
    return counts


def fr_rank_tokens(counts, freq_ranked_ids=None, stream=None):
    """All ids by count descending, equal counts by lower id (int32 [V])."""
    _dev(counts, torch.int64, "counts")
    V = counts.numel()
    if freq_ranked_ids is None:
        freq_ranked_ids = torch.empty(V, dtype=torch.int32, device=counts.device)
    _check(lib().fr_rank_tokens(_ptr(counts), V, _ptr(_dev(freq_ranked_ids, torch.int32, "freq_ranked_ids")),
                                _stream(stream)), "fr_rank_tokens")
    return freq_ranked_ids


def fr_tiled_bytes(V_sub: int, d: int) -> int:
    return int(lib().fr_tiled_bytes(V_sub, d))


def fr_build_subset_tiled(W_full, freq_ranked_ids, V_sub: int, W_tiled=None, idx_map=None,
                          dev_error_flag=None, stream=None):
    """Eq. 3 into the private tiled layout (see frspec.h).  Returns (W_tiled, idx_map);
    W_tiled is a flat bf16 tensor of fr_tiled_bytes(V_sub, d) / 2 elements."""
    _bf16_matrix(W_full, "W_full")
    V, d = W_full.shape
    n = fr_tiled_bytes(V_sub, d)
    if n == 0:
        raise ValueError("the tiled layout needs d to be a multiple of 128")
    if W_tiled is None:
        W_tiled = torch.empty(n // 2, dtype=W_full.dtype, device=W_full.device)
    if idx_map is None:
        idx_map = torch.empty(V_sub, dtype=torch.int32, device=W_full.device)
    if W_tiled.numel() * W_tiled.element_size() < n or not W_tiled.is_contiguous():
        raise ValueError("W_tiled is too small")
    _check(lib().fr_build_subset_tiled(_ptr(W_full), V, d, _ptr(freq_ranked_ids), V_sub, _ptr(W_tiled),
                                       _ptr(idx_map), _ptr(dev_error_flag), _stream(stream)),
           "fr_build_subset_tiled")
    return W_tiled, idx_map


def fr_draft_topk_tiled(H, W_tiled, idx_map, V_sub: int, k: int, workspace, token_ids=None, logp=None,
                        stream=None, tuning=None):
    """fr_draft_topk on a W_sub in the tiled layout."""
    _bf16_matrix(H, "H")
    M, d = H.shape
    if W_tiled.numel() * W_tiled.element_size() < fr_tiled_bytes(V_sub, d) or fr_tiled_bytes(V_sub, d) == 0:
        raise ValueError("W_tiled does not hold V_sub rows of d elements in the tiled layout")
    if token_ids is None:
        token_ids = torch.empty((M, k), dtype=torch.int32, device=H.device)
    if logp is None:
        logp = torch.empty((M, k), dtype=torch.float32, device=H.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    if tuning is None:
        st = lib().fr_draft_topk_tiled(_ptr(H), M, d, _ptr(W_tiled), _ptr(idx_map), V_sub, k, _ptr(token_ids),
                                       _ptr(logp), _ptr(workspace), ws_bytes, _stream(stream))
    else:
        st = lib().fr_draft_topk_tiled_tuned(_ptr(H), M, d, _ptr(W_tiled), _ptr(idx_map), V_sub, k, _ptr(token_ids),
                                             _ptr(logp), _ptr(workspace), ws_bytes, _stream(stream),
                                             ctypes.byref(tuning))
    _check(st, "fr_draft_topk_tiled")
    return token_ids, logp


def _dev(t, dtype, name):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError(f"{name} must be a contiguous CUDA tensor of {dtype}")
    return t


def fr_beam_expand(logp, token_ids, node_score, node_hist, width: int, hist_score, hist_token, hist_parent,
                   hist_offset: int, next_score=None, next_token=None, next_hist=None, stream=None):
    """One beam-search draft step (Section 2): appends the M*k candidates to the history at
    hist_offset and returns (next_score, next_token, next_hist) of the `width` best."""
    M, k = logp.shape
    _dev(logp, torch.float32, "logp")
    _dev(token_ids, torch.int32, "token_ids")
    _dev(node_score, torch.float32, "node_score")
    _dev(node_hist, torch.int32, "node_hist")
    _dev(hist_score, torch.float32, "hist_score")
    _dev(hist_token, torch.int32, "hist_token")
    _dev(hist_parent, torch.int32, "hist_parent")
    if token_ids.shape != (M, k) or node_score.numel() != M or node_hist.numel() != M:
        raise ValueError("token_ids must be [M, k]; node_score and node_hist [M]")
    if min(hist_score.numel(), hist_token.numel(), hist_parent.numel()) < hist_offset + M * k:
        raise ValueError("history arrays are too short for hist_offset + M*k entries")
    if next_score is None:
        next_score = torch.empty(width, dtype=torch.float32, device=logp.device)
    if next_token is None:
        next_token = torch.empty(width, dtype=torch.int32, device=logp.device)
    if next_hist is None:
        next_hist = torch.empty(width, dtype=torch.int32, device=logp.device)
    if min(next_score.numel(), next_token.numel(), next_hist.numel()) < width:
        raise ValueError("next_* must hold `width` entries")
    _check(lib().fr_beam_expand(_ptr(logp), _ptr(token_ids), M, k, _ptr(node_score), _ptr(node_hist), width,
                                _ptr(hist_score), _ptr(hist_token), _ptr(hist_parent), hist_offset,
                                _ptr(_dev(next_score, torch.float32, "next_score")),
                                _ptr(_dev(next_token, torch.int32, "next_token")),
                                _ptr(_dev(next_hist, torch.int32, "next_hist")), _stream(stream)),
           "fr_beam_expand")
    return next_score, next_token, next_hist


def fr_draft_step(H, W_sub, idx_map, k: int, node_score, node_hist, width: int, hist_score, hist_token,
                  hist_parent, hist_offset: int, workspace, token_ids=None, logp=None, next_score=None,
                  next_token=None, next_hist=None, stream=None):
    """The draft LM head on the nodes of a draft step and the beam-search expansion, one call
    (one launch for M <= 16, k <= 16).  Returns (token_ids, logp, next_score, next_token, next_hist)."""
    _bf16_matrix(H, "H")
    _bf16_matrix(W_sub, "W_sub")
    M, d = H.shape
    dev = H.device
    if token_ids is None:
        token_ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    if logp is None:
        logp = torch.empty((M, k), dtype=torch.float32, device=dev)
    if next_score is None:
        next_score = torch.empty(width, dtype=torch.float32, device=dev)
    if next_token is None:
        next_token = torch.empty(width, dtype=torch.int32, device=dev)
    if next_hist is None:
        next_hist = torch.empty(width, dtype=torch.int32, device=dev)
    for t, dt, name in ((node_score, torch.float32, "node_score"), (node_hist, torch.int32, "node_hist"),
                        (hist_score, torch.float32, "hist_score"), (hist_token, torch.int32, "hist_token"),
                        (hist_parent, torch.int32, "hist_parent"), (next_score, torch.float32, "next_score"),
                        (next_token, torch.int32, "next_token"), (next_hist, torch.int32, "next_hist")):
        _dev(t, dt, name)
    if node_score.numel() < M or node_hist.numel() < M:
        raise ValueError("node_score and node_hist must hold M entries")
    if min(hist_score.numel(), hist_token.numel(), hist_parent.numel()) < hist_offset + M * k:
        raise ValueError("history arrays are too short for hist_offset + M*k entries")
    if min(next_score.numel(), next_token.numel(), next_hist.numel()) < width:
        raise ValueError("next_* must hold `width` entries")
    _check(lib().fr_draft_step(_ptr(H), M, d, _ptr(W_sub), _ptr(idx_map), W_sub.shape[0], k, _ptr(node_score),
                               _ptr(node_hist), width, _ptr(hist_score), _ptr(hist_token), _ptr(hist_parent),
                               hist_offset, _ptr(token_ids), _ptr(logp), _ptr(next_score), _ptr(next_token),
                               _ptr(next_hist), _ptr(workspace), workspace.numel() * workspace.element_size(),
                               _stream(stream)), "fr_draft_step")
    return token_ids, logp, next_score, next_token, next_hist


def fr_tree_select(hist_score, hist_token, hist_parent, N: int, K: int, stream=None, out=None):
    """The draft tree (Section 2): the K best of the first N history entries.  Returns
    (sel_index, sel_token, sel_parent, sel_depth, tree_mask[K, K] uint8); `out`, if given, is
    that tuple preallocated (int32 [K] four times, uint8 [K, K])."""
    _dev(hist_score, torch.float32, "hist_score")
    _dev(hist_token, torch.int32, "hist_token")
    _dev(hist_parent, torch.int32, "hist_parent")
    if min(hist_score.numel(), hist_token.numel(), hist_parent.numel()) < N:
        raise ValueError("history arrays are shorter than N")
    dev = hist_score.device
    if out is not None:
        *out, mask = out
        for t in out:
            _dev(t, torch.int32, "out")
            if t.numel() < K:
                raise ValueError("selection outputs are shorter than K")
        _dev(mask, torch.uint8, "tree_mask")
        if mask.numel() < K * K:
            raise ValueError("tree_mask is smaller than K * K")
    else:
        out = [torch.empty(K, dtype=torch.int32, device=dev) for _ in range(4)]
        mask = torch.empty((K, K), dtype=torch.uint8, device=dev)
    _check(lib().fr_tree_select(_ptr(hist_score), _ptr(hist_token), _ptr(hist_parent), N, K, _ptr(out[0]),
                                _ptr(out[1]), _ptr(out[2]), _ptr(out[3]), _ptr(mask), _stream(stream)),
           "fr_tree_select")
    return out[0], out[1], out[2], out[3], mask


def fr_calib_copy(dst, src, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().fr_calib_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "fr_calib_copy")


def fr_calib_read(src, sink, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().fr_calib_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "fr_calib_read")
