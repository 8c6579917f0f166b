"""Pins of the draft-step glue oracle (beam expansion, draft-tree selection) to things other
than itself: a hand-worked example, numpy's sort, brute-force ancestor sets, closed forms.

Section 2 of the paper describes the procedure in words only (beam search on the softmax
output, K best of the search history, ancestral-path mask); the readings are listed in the
oracle's header.
"""

import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "beam_two_steps.txt")


def _two_step_history():
    hs = np.full(9, np.nan, dtype=np.float32)
    ht = np.full(9, -7, dtype=np.int32)
    hp = np.full(9, -7, dtype=np.int32)
    n0 = oracle.beam_expand(np.array([[-1, -2, -4]], np.float32), np.array([[10, 11, 12]], np.int32),
                            np.array([0], np.float32), np.array([-1], np.int32), 2, hs, ht, hp, 0)
    n1 = oracle.beam_expand(np.array([[-0.5, -1.5, -3], [-0.25, -1, -5]], np.float32),
                            np.array([[20, 21, 22], [30, 31, 32]], np.int32), n0[0], n0[2], 2, hs, ht, hp, 3)
    return hs, ht, hp, n0, n1


def test_hand_worked_two_step_example():
    hs, ht, hp, n0, n1 = _two_step_history()
    assert n0[0].tolist() == [-1.0, -2.0] and n0[1].tolist() == [10, 11] and n0[2].tolist() == [0, 1]
    assert n1[0].tolist() == [-1.5, -2.25] and n1[1].tolist() == [20, 30] and n1[2].tolist() == [3, 6]
    assert hs.tolist() == [-1, -2, -4, -1.5, -2.5, -4, -2.25, -3, -7]
    assert ht.tolist() == [10, 11, 12, 20, 21, 22, 30, 31, 32]
    assert hp.tolist() == [-1, -1, -1, 0, 0, 0, 1, 1, 1]
    rows = [l for l in open(GOLDEN).read().splitlines() if l and not l.startswith("#")]
    for line in rows:
        if line.startswith("mask5"):
            want = np.array([[int(ch) for ch in word] for word in line.split("|")[1].split()], dtype=np.uint8)
            assert np.array_equal(oracle.tree_select(hs, ht, hp, 5)[4], want)
            continue
        K, idx, tok, par, dep = [np.array(f.split(), dtype=np.int64) for f in line.split("|")]
        got = oracle.tree_select(hs, ht, hp, int(K[0]))
        assert got[0].tolist() == idx.tolist()
        assert got[1].tolist() == tok.tolist()
        assert got[2].tolist() == par.tolist()
        assert got[3].tolist() == dep.tolist()


def _random_history(rng, n_roots, n, quantised):
    """A random forest in append order whose scores never rise along a path."""
    parent = np.empty(n, dtype=np.int32)
    score = np.empty(n, dtype=np.float32)
    for i in range(n):
        parent[i] = -1 if i < n_roots else int(rng.integers(-1, i))
        step = -float(rng.integers(0, 6)) / 4 if quantised else -float(rng.exponential(1.0))
        score[i] = np.float32((0.0 if parent[i] < 0 else score[parent[i]]) + np.float32(step))
    token = rng.integers(0, 128256, size=n).astype(np.int32)
    return score, token, parent


def _ancestors(parent, i):
    out = []
    while parent[i] >= 0:
        i = parent[i]
        out.append(i)
    return out


@pytest.mark.parametrize("seed,n,K,quantised", [(0, 40, 12, True), (1, 606, 60, False), (2, 606, 60, True),
                                                (3, 100, 100, True), (4, 1, 1, False), (5, 2000, 128, True)])
def test_tree_select_against_numpy_and_brute_force(seed, n, K, quantised):
    rng = np.random.default_rng([20250214, 77, seed])
    score, token, parent = _random_history(rng, min(n, 10), n, quantised)
    idx, tok, par, dep, mask = oracle.tree_select(score, token, parent, K)
    # numpy's stable sort on the negated score keeps lower indices first among equals
    want = np.sort(np.argsort(-score.astype(np.float64), kind="stable")[:K])
    assert np.array_equal(idx, want)
    assert np.array_equal(tok, token[want])
    pos = {int(h): p for p, h in enumerate(want)}
    for p, h in enumerate(want):
        anc = _ancestors(parent, int(h))
        assert all(a in pos for a in anc)                      # closed under ancestors
        assert par[p] == (pos[anc[0]] if anc else -1)
        assert dep[p] == len(anc)
        row = np.zeros(K, dtype=np.uint8)
        row[[pos[a] for a in anc] + [p]] = 1
        assert np.array_equal(mask[p], row)
    # structure: unit diagonal, nothing above it, a row is its parent's row plus itself
    assert np.array_equal(np.diag(mask), np.ones(K, dtype=np.uint8))
    assert not np.triu(mask, 1).any()
    assert np.array_equal(mask.sum(axis=1), dep + 1)


def test_chain_gives_full_lower_triangle():
    n = 17
    score = -np.arange(1, n + 1, dtype=np.float32)
    parent = np.arange(-1, n - 1, dtype=np.int32)
    idx, tok, par, dep, mask = oracle.tree_select(score, np.arange(n, dtype=np.int32), parent, n)
    assert idx.tolist() == list(range(n)) and par.tolist() == list(range(-1, n - 1))
    assert dep.tolist() == list(range(n))
    assert np.array_equal(mask, np.tril(np.ones((n, n), dtype=np.uint8)))


@pytest.mark.parametrize("seed,M,k,width", [(0, 1, 10, 10), (1, 10, 10, 10), (2, 10, 10, 100), (3, 16, 4, 7),
                                            (4, 3, 64, 50)])
def test_expand_against_numpy(seed, M, k, width):
    rng = np.random.default_rng([20250214, 78, seed])
    # quantised log-probabilities: plenty of exactly equal cumulative scores
    logp = (-rng.integers(0, 12, size=(M, k)) / 4).astype(np.float32)
    tok = rng.integers(0, 128256, size=(M, k)).astype(np.int32)
    node_score = (-rng.integers(0, 8, size=M) / 2).astype(np.float32)
    node_hist = rng.integers(-1, 50, size=M).astype(np.int32)
    off = 50
    hs = np.zeros(off + M * k, np.float32)
    ht = np.zeros(off + M * k, np.int32)
    hp = np.zeros(off + M * k, np.int32)
    ns, nt, nh = oracle.beam_expand(logp, tok, node_score, node_hist, width, hs, ht, hp, off)
    cand = (node_score[:, None] + logp).astype(np.float32).reshape(-1)
    assert np.array_equal(hs[off:], cand) and not hs[:off].any()
    assert np.array_equal(ht[off:], tok.reshape(-1))
    assert np.array_equal(hp[off:], np.repeat(node_hist, k))
    order = np.argsort(-cand.astype(np.float64), kind="stable")[:width]
    assert np.array_equal(ns, cand[order])
    assert np.array_equal(nt, tok.reshape(-1)[order])
    assert np.array_equal(nh, off + order)


def test_cumulative_score_is_log_of_path_probability():
    # closed form: exp(score) of a history entry = product of the probabilities on its path
    rng = np.random.default_rng([20250214, 79])
    depth, width, k = 4, 3, 5
    hs = np.zeros(k + (depth - 1) * width * k, np.float32)
    ht = np.zeros_like(hs, dtype=np.int32)
    hp = np.zeros_like(hs, dtype=np.int32)
    probs_of = {}
    node_score, node_hist, off = np.zeros(1, np.float32), np.full(1, -1, np.int32), 0
    for step in range(depth):
        M = len(node_score)
        p = rng.dirichlet(np.ones(k), size=M)
        logp = np.log(p).astype(np.float32)
        for m in range(M):
            for j in range(k):
                probs_of[off + m * k + j] = p[m, j]
        tok = rng.integers(0, 1000, size=(M, k)).astype(np.int32)
        node_score, _, node_hist = oracle.beam_expand(logp, tok, node_score, node_hist, min(width, M * k),
                                                      hs, ht, hp, off)
        off += M * k
    for i in range(off):
        path = [i] + _ancestors(hp, i)
        assert np.exp(hs[i]) == pytest.approx(np.prod([probs_of[a] for a in path]), rel=1e-5)


def test_argument_errors():
    hs = np.zeros(4, np.float32)
    hi = np.zeros(4, np.int32)
    with pytest.raises(oracle.OracleError):
        oracle.tree_select(hs, hi, np.array([-1, 0, 1, 5], np.int32), 2)      # parent after child
    with pytest.raises(oracle.OracleError):
        oracle.tree_select(hs, hi, np.full(4, -1, np.int32), 5)              # K > N
    with pytest.raises(oracle.OracleError):
        oracle.beam_expand(np.zeros((1, 2), np.float32), np.zeros((1, 2), np.int32), np.zeros(1, np.float32),
                           np.zeros(1, np.int32), 3, hs, hi, hi.copy(), 0)   # width > M*k
