"""Pins of the corpus-statistics oracle (token counting, frequency ranking; Section 3.2) to
numpy's bincount / lexsort, to closed forms and to the synthetic ranking generator."""

import numpy as np
import pytest

import oracle
from synth import zipf_ranking


def test_counts_equal_bincount_and_skip_bad_ids():
    rng = np.random.default_rng([20250214, 95])
    V = 5000
    tokens = rng.zipf(1.3, size=200000).astype(np.int64) - 1
    tokens = np.where(tokens < V + 50, tokens, rng.integers(0, V, size=tokens.size)).astype(np.int32)
    tokens[::997] = -3
    counts, bad = oracle.count_tokens(tokens, V)
    good = tokens[(tokens >= 0) & (tokens < V)]
    assert np.array_equal(counts, np.bincount(good, minlength=V))
    assert bad == tokens.size - good.size and bad > 0
    # accumulation over two halves = one pass
    c2, _ = oracle.count_tokens(tokens[:70001], V)
    c2, _ = oracle.count_tokens(tokens[70001:], V, c2)
    assert np.array_equal(c2, counts)


def test_ranking_equals_lexsort_with_ties_by_lower_id():
    rng = np.random.default_rng([20250214, 96])
    counts = rng.integers(0, 40, size=20000).astype(np.int64)       # many equal counts
    got = oracle.rank_tokens(counts)
    want = np.lexsort((np.arange(counts.size), -counts)).astype(np.int32)
    assert np.array_equal(got, want)
    assert np.array_equal(np.sort(got), np.arange(counts.size))     # a permutation
    assert (np.diff(counts[got]) <= 0).all()                        # counts never rise


def test_closed_forms():
    V = 1000
    assert np.array_equal(oracle.rank_tokens(np.zeros(V, np.int64)), np.arange(V))          # all tied: by id
    assert np.array_equal(oracle.rank_tokens(np.arange(V, dtype=np.int64)), np.arange(V)[::-1])
    big = np.array([1 << 40, (1 << 40) + 1, 5, (1 << 62)], dtype=np.int64)                  # beyond 32 bits
    assert oracle.rank_tokens(big).tolist() == [3, 1, 0, 2]


def test_counting_then_ranking_reproduces_the_synthetic_generator():
    # the generator draws counts and ranks them itself; a token stream with exactly those counts,
    # counted and ranked by the oracle, must give the same ranking (same tie rule)
    V = 3000
    ranked, counts = zipf_ranking(V, 1.1, 10 ** 5, 7)
    stream = np.repeat(np.arange(V, dtype=np.int32), counts)
    np.random.default_rng(1).shuffle(stream)
    c, bad = oracle.count_tokens(stream, V)
    assert bad == 0 and np.array_equal(c, counts)
    assert np.array_equal(oracle.rank_tokens(c), ranked)


def test_argument_errors():
    with pytest.raises(oracle.OracleError):
        oracle.rank_tokens(np.zeros(0, np.int64))
