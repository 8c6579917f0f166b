"""Deterministic generators for the draft-head workloads.

Shapes follow the models the paper evaluates (Section 4.1, "Models":
Llama-3-8B with a 128k vocabulary, Qwen-2-7B with a 152k vocabulary) and the
subset sizes it sweeps (Section 4.2: 8k, 16k, 32k, 64k).  The real LM heads,
EAGLE-2 hidden states and corpus frequency tables are not available, so:

* ``W_full``  : fp32 N(0, 0.02^2) rounded to bf16 (round-to-nearest-even),
* ``H``       : fp32 N(0, 1) rounded to bf16,
* ranking     : token counts drawn from a Zipf(s) law over a seeded random
                permutation of the ids, then sorted by (count desc, id asc).
                Section 3.2 reports that a quarter of the ids cover about 95%
                of corpus occurrences; Zipf(1.1) over 128256 ids puts 94% of
                the mass in the top 32768 ranks.

Every array is a pure function of (BASE_SEED, config index, stream id) so the
oracle and the GPU path see identical bytes.
"""

from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250214

_STREAM_W = 0
_STREAM_H = 1
_STREAM_PERM = 2
_STREAM_COUNTS = 3

# Rows generated per independent sub-stream of W.  Fixed, so the bytes do not
# depend on how a caller chunks the work.
_W_BLOCK_ROWS = 4096


@dataclass(frozen=True)
class DraftHeadConfig:
    """One synthetic draft-step workload."""

    name: str
    index: int          # seeds the generators
    d: int              # hidden size
    V: int              # full vocabulary
    V_sub: int          # |V_high|
    M: int              # rows of H (tree nodes expanded in one draft step)
    k: int              # candidates kept per row
    zipf_s: float
    n_tokens: int       # corpus size the counts are drawn from


CONFIGS = {
    # small case the oracle finishes in milliseconds
    "tiny": DraftHeadConfig("tiny", 0, 256, 8192, 2048, 4, 4, 1.1, 10**6),
    # Llama-3-8B-shaped draft step (depth-step of an EAGLE-2 tree, 10 nodes)
    "llama3_8b": DraftHeadConfig("llama3_8b", 1, 4096, 128256, 32768, 10, 10, 1.1, 10**8),
    # Qwen-2.5-7B-shaped, six depths of ten nodes batched
    "qwen25_7b": DraftHeadConfig("qwen25_7b", 3, 3584, 152064, 32768, 60, 10, 1.0, 10**8),
    # many requests drafted together
    "batched256": DraftHeadConfig("batched256", 4, 4096, 128256, 32768, 256, 10, 1.1, 10**8),
}

# Vocabulary-subset sweep of Section 4.2 at the Llama-3-8B shape.
SWEEP_V_SUB = (8192, 16384, 32768, 65536, 128256)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 patterns.

    Inputs are finite by construction; NaN payloads are not treated specially.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact: the pattern is the upper half)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(config_index: int, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, int(config_index), int(stream), int(block)])


def _weights_block(V, d, config_index, std, b0, lo, hi, out):
    b1 = min(b0 + _W_BLOCK_ROWS, V)
    g = _rng(config_index, _STREAM_W, b0 // _W_BLOCK_ROWS)
    blk = g.standard_normal((b1 - b0, d), dtype=np.float32)
    blk *= np.float32(std)
    take = min(b1, hi) - b0
    out[b0 - lo:b0 - lo + take] = f32_to_bf16_bits(blk[:take])


def make_weights(V: int, d: int, config_index: int, std: float = 0.02,
                 rows: slice | None = None, threads: int | None = None) -> np.ndarray:
    """bf16 bit patterns of W_full [V, d], row-major, entries ~ N(0, std^2).

    Each block of 4096 rows has its own generator stream, so the bytes depend neither on
    ``rows`` (a row range starting on a block boundary, used to build a large W piecewise)
    nor on ``threads`` (blocks are filled concurrently).
    """
    lo, hi = (0, V) if rows is None else (rows.start or 0, V if rows.stop is None else rows.stop)
    if lo % _W_BLOCK_ROWS:
        raise ValueError("row range must start on a generator block boundary")
    out = np.empty((hi - lo, d), dtype=np.uint16)
    starts = list(range(lo, hi, _W_BLOCK_ROWS))
    if threads is None:
        threads = min(8, os.cpu_count() or 1)
    if threads <= 1 or len(starts) <= 1:
        for b0 in starts:
            _weights_block(V, d, config_index, std, b0, lo, hi, out)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda b0: _weights_block(V, d, config_index, std, b0, lo, hi, out), starts))
    return out


def make_hidden(M: int, d: int, config_index: int, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns of H [M, d], entries ~ N(0, std^2)."""
    g = _rng(config_index, _STREAM_H)
    h = g.standard_normal((M, d), dtype=np.float32) * np.float32(std)
    return f32_to_bf16_bits(h)


def zipf_ranking(V: int, s: float, n_tokens: int, config_index: int):
    """Frequency-ranked id list standing in for corpus statistics.

    Rank j (1-based) has probability proportional to j^-s; the token at rank j
    is ``perm[j-1]`` for a seeded permutation of the ids.  ``n_tokens`` draws
    give per-id counts; ids are then ordered by count descending, equal counts
    by lower id (many tail ids tie, ids never drawn sort last).

    Returns (freq_ranked_ids int32 [V], counts_by_id int64 [V]).
    """
    perm = _rng(config_index, _STREAM_PERM).permutation(V)
    j = np.arange(1, V + 1, dtype=np.float64)
    p = j ** (-float(s))
    p /= p.sum()
    counts_by_rank = _rng(config_index, _STREAM_COUNTS).multinomial(int(n_tokens), p)
    counts_by_id = np.zeros(V, dtype=np.int64)
    counts_by_id[perm] = counts_by_rank
    ids = np.arange(V, dtype=np.int64)
    order = np.lexsort((ids, -counts_by_id))   # last key is primary
    return order.astype(np.int32), counts_by_id


def make_exact_case(V: int, d: int, M: int, seed: int, w_levels: int = 3, h_levels: int = 2):
    """Inputs on which every summation order gives the same bits.

    W entries are small integers in [-w_levels, w_levels], H entries integers
    in [-h_levels, h_levels] (all exactly representable in bf16).  Every
    partial sum of products is an integer far below 2^24, hence exact in fp32
    whatever the order or fusion of the accumulation.

    Returns (W_bits uint16 [V,d], H_bits uint16 [M,d], W_int int64, H_int int64).
    """
    g = np.random.default_rng([BASE_SEED, 9000, int(seed)])
    W_int = g.integers(-w_levels, w_levels + 1, size=(V, d), dtype=np.int64)
    H_int = g.integers(-h_levels, h_levels + 1, size=(M, d), dtype=np.int64)
    W_bits = f32_to_bf16_bits(W_int.astype(np.float32))
    H_bits = f32_to_bf16_bits(H_int.astype(np.float32))
    return W_bits, H_bits, W_int, H_int
