"""ctypes front end of the CPU oracle (``frspec_oracle.c``, ``beam_oracle.c``, ``freq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.

Arrays are numpy: bf16 tensors travel as ``uint16`` bit patterns.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "frspec_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "beam_oracle.c"), os.path.join(_HERE, "freq_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle.so")
# A differently built copy of the same sources (the sanitizer build of the test suite) can stand in.
_LIB_OVERRIDE = os.environ.get("FRSPEC_ORACLE_SO")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math).  Returns the .so path."""
    if _LIB_OVERRIDE and not force:
        return _LIB_OVERRIDE
    stale = not os.path.exists(_LIB) or any(os.path.getmtime(_LIB) < os.path.getmtime(src) for src in _SRCS)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_build_subset.argtypes = [vp, i64, i64, vp, i64, vp, vp]
        lib.oracle_logits_f32.argtypes = [vp, i64, i64, vp, i64, vp]
        lib.oracle_logits_f64.argtypes = [vp, i64, i64, vp, i64, vp]
        lib.oracle_log_softmax.argtypes = [vp, i64, i64, vp, vp]
        lib.oracle_topk.argtypes = [vp, i64, i64, vp, i32, vp, vp]
        lib.oracle_draft_topk.argtypes = [vp, i64, i64, vp, vp, i64, i32, vp, vp, vp]
        lib.oracle_full_topk.argtypes = [vp, i64, i64, vp, i64, i32, vp, vp, vp]
        lib.oracle_num_threads.argtypes = []
        lib.oracle_beam_expand.argtypes = [vp, vp, i64, i32, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp]
        lib.oracle_tree_select.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, vp, vp]
        lib.oracle_count_tokens.argtypes = [vp, i64, i64, vp, vp]
        lib.oracle_rank_tokens.argtypes = [vp, i64, vp]
        for name in ("oracle_count_tokens", "oracle_rank_tokens"):
            getattr(lib, name).restype = ctypes.c_int
        for name in ("oracle_build_subset", "oracle_logits_f32", "oracle_logits_f64",
                     "oracle_log_softmax", "oracle_topk", "oracle_draft_topk",
                     "oracle_full_topk", "oracle_num_threads", "oracle_beam_expand",
                     "oracle_tree_select"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    pass


def _check(status: int, what: str) -> None:
    if status != 0:
        raise OracleError(f"{what} failed with status {status}")


def _u16(a, shape_len):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    assert a.ndim == shape_len
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def build_subset(W_full, freq_ranked_ids, V_sub):
    """Eq. 3.  Returns (W_sub uint16 [V_sub, d], idx_map int32 [V_sub])."""
    W_full = _u16(W_full, 2)
    ids = np.ascontiguousarray(freq_ranked_ids, dtype=np.int32)
    V, d = W_full.shape
    if not (1 <= V_sub <= min(V, ids.size)):
        raise OracleError("V_sub out of range")
    W_sub = np.empty((V_sub, d), dtype=np.uint16)
    idx_map = np.empty(V_sub, dtype=np.int32)
    _check(_load().oracle_build_subset(_p(W_full), V, d, _p(ids), V_sub, _p(W_sub), _p(idx_map)),
           "oracle_build_subset")
    return W_sub, idx_map


def logits_f32(H, W):
    """fp32-accumulated logits z [M, rows]."""
    H, W = _u16(H, 2), _u16(W, 2)
    M, d = H.shape
    rows = W.shape[0]
    assert W.shape[1] == d
    z = np.empty((M, rows), dtype=np.float32)
    _check(_load().oracle_logits_f32(_p(H), M, d, _p(W), rows, _p(z)), "oracle_logits_f32")
    return z


def logits_f64(H, W):
    """fp64-accumulated logits [M, rows] (the exact value up to fp64 rounding)."""
    H, W = _u16(H, 2), _u16(W, 2)
    M, d = H.shape
    rows = W.shape[0]
    assert W.shape[1] == d
    z = np.empty((M, rows), dtype=np.float64)
    _check(_load().oracle_logits_f64(_p(H), M, d, _p(W), rows, _p(z)), "oracle_logits_f64")
    return z


def log_softmax(z):
    """Returns (logp float32 [M, rows], logZ float64 [M])."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    M, rows = z.shape
    logp = np.empty_like(z)
    logZ = np.empty(M, dtype=np.float64)
    _check(_load().oracle_log_softmax(_p(z), M, rows, _p(logp), _p(logZ)), "oracle_log_softmax")
    return logp, logZ


def topk(z, idx_map, k):
    """Returns (token_ids int32 [M, k], positions int32 [M, k])."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    M, rows = z.shape
    im = None if idx_map is None else np.ascontiguousarray(idx_map, dtype=np.int32)
    ids = np.empty((M, k), dtype=np.int32)
    pos = np.empty((M, k), dtype=np.int32)
    _check(_load().oracle_topk(_p(z), M, rows, _p(im), k, _p(ids), _p(pos)), "oracle_topk")
    return ids, pos


def draft_topk(H, W_sub, idx_map, k, want_logits=False):
    """Eq. 4, candidate selection, id translation.

    Returns (token_ids int32 [M,k], logp float32 [M,k]) and, if asked, the
    full fp32 logits [M, V_sub] as a third element.
    """
    H, W_sub = _u16(H, 2), _u16(W_sub, 2)
    M, d = H.shape
    V_sub = W_sub.shape[0]
    assert W_sub.shape[1] == d
    im = None if idx_map is None else np.ascontiguousarray(idx_map, dtype=np.int32)
    ids = np.empty((M, k), dtype=np.int32)
    logp = np.empty((M, k), dtype=np.float32)
    z = np.empty((M, V_sub), dtype=np.float32) if want_logits else None
    _check(_load().oracle_draft_topk(_p(H), M, d, _p(W_sub), _p(im), V_sub, k,
                                     _p(ids), _p(logp), _p(z)), "oracle_draft_topk")
    return (ids, logp, z) if want_logits else (ids, logp)


def full_topk(H, W_full, k, want_logits=False):
    """Eq. 2 with the same candidate selection; position == id."""
    H, W_full = _u16(H, 2), _u16(W_full, 2)
    M, d = H.shape
    V = W_full.shape[0]
    ids = np.empty((M, k), dtype=np.int32)
    logp = np.empty((M, k), dtype=np.float32)
    z = np.empty((M, V), dtype=np.float32) if want_logits else None
    _check(_load().oracle_full_topk(_p(H), M, d, _p(W_full), V, k, _p(ids), _p(logp), _p(z)),
           "oracle_full_topk")
    return (ids, logp, z) if want_logits else (ids, logp)


def beam_expand(logp, token_ids, node_score, node_hist, width, hist_score, hist_token, hist_parent,
                hist_offset):
    """One draft step of the beam search (Section 2).  Appends the M*k candidates to the history
    arrays (in place, at hist_offset) and returns (next_score, next_token, next_hist) of the
    `width` best."""
    logp = np.ascontiguousarray(logp, dtype=np.float32)
    token_ids = np.ascontiguousarray(token_ids, dtype=np.int32)
    node_score = np.ascontiguousarray(node_score, dtype=np.float32)
    node_hist = np.ascontiguousarray(node_hist, dtype=np.int32)
    M, k = logp.shape
    assert token_ids.shape == (M, k) and node_score.shape == (M,) and node_hist.shape == (M,)
    for a, dt in ((hist_score, np.float32), (hist_token, np.int32), (hist_parent, np.int32)):
        assert a.dtype == dt and a.flags.c_contiguous and a.shape[0] >= hist_offset + M * k
    next_score = np.empty(width, dtype=np.float32)
    next_token = np.empty(width, dtype=np.int32)
    next_hist = np.empty(width, dtype=np.int32)
    _check(_load().oracle_beam_expand(_p(logp), _p(token_ids), M, k, _p(node_score), _p(node_hist), width,
                                      _p(hist_score), _p(hist_token), _p(hist_parent), hist_offset,
                                      _p(next_score), _p(next_token), _p(next_hist)), "oracle_beam_expand")
    return next_score, next_token, next_hist


def tree_select(hist_score, hist_token, hist_parent, K):
    """The draft tree: the K best history entries in history order, with the position of each
    one's parent, its depth and the ancestor mask (Section 2).  Returns (sel_index, sel_token,
    sel_parent, sel_depth, tree_mask[K, K] uint8)."""
    hist_score = np.ascontiguousarray(hist_score, dtype=np.float32)
    hist_token = np.ascontiguousarray(hist_token, dtype=np.int32)
    hist_parent = np.ascontiguousarray(hist_parent, dtype=np.int32)
    N = hist_score.shape[0]
    assert hist_token.shape == (N,) and hist_parent.shape == (N,)
    sel_index = np.empty(K, dtype=np.int32)
    sel_token = np.empty(K, dtype=np.int32)
    sel_parent = np.empty(K, dtype=np.int32)
    sel_depth = np.empty(K, dtype=np.int32)
    mask = np.empty((K, K), dtype=np.uint8)
    _check(_load().oracle_tree_select(_p(hist_score), _p(hist_token), _p(hist_parent), N, K, _p(sel_index),
                                      _p(sel_token), _p(sel_parent), _p(sel_depth), _p(mask)),
           "oracle_tree_select")
    return sel_index, sel_token, sel_parent, sel_depth, mask


def count_tokens(tokens, V, counts=None):
    """Corpus-level token statistics (Section 3.2): adds the occurrences of every id of the
    stream to counts (int64 [V], created zeroed if not given).  Returns (counts, n_bad) where
    n_bad is the number of ids outside [0, V) that were skipped."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    if counts is None:
        counts = np.zeros(V, dtype=np.int64)
    assert counts.dtype == np.int64 and counts.shape == (V,) and counts.flags.c_contiguous
    bad = ctypes.c_int64(0)
    _check(_load().oracle_count_tokens(_p(tokens), tokens.size, V, _p(counts), ctypes.addressof(bad)),
           "oracle_count_tokens")
    return counts, int(bad.value)


def rank_tokens(counts):
    """All ids ordered by count descending, equal counts by lower id: the frequency ranking
    from which V_high is taken (Section 3.2)."""
    counts = np.ascontiguousarray(counts, dtype=np.int64)
    out = np.empty(counts.shape[0], dtype=np.int32)
    _check(_load().oracle_rank_tokens(_p(counts), counts.shape[0], _p(out)), "oracle_rank_tokens")
    return out
