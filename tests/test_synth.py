"""The input generators: determinism, bf16 rounding, ranking validity, long-tail shape."""

import os

import numpy as np
import torch

from synth import (bf16_bits_to_f32, f32_to_bf16_bits, make_exact_case, make_hidden,
                   make_weights, zipf_ranking)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_long_tail():
    paper, zipf = {}, []
    for line in open(os.path.join(GOLDEN, "long_tail.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "zipf":
            zipf.append((int(t[1]), int(t[2]), float(t[3]), float(t[4])))
        else:
            paper[t[0]] = float(t[1])
    return paper, zipf


def test_bf16_rounding_is_rne_and_matches_torch():
    g = np.random.default_rng(0)
    x = (g.standard_normal(100000) * 3).astype(np.float32)
    ours = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    # exact tie cases: 1 + 2^-8 is halfway between two bf16 values -> even mantissa
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert f32_to_bf16_bits(ties).tolist() == [0x3F80, 0x3F82]
    assert np.array_equal(bf16_bits_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_weights_are_deterministic_and_chunk_independent():
    a = make_weights(9000, 32, 0)
    b = make_weights(9000, 32, 0)
    assert np.array_equal(a, b)
    part = make_weights(9000, 32, 0, rows=slice(4096, 9000))
    assert np.array_equal(part, a[4096:])
    c = make_weights(9000, 32, 1)
    assert not np.array_equal(a, c)
    f = bf16_bits_to_f32(a)
    assert abs(f.std() - 0.02) < 5e-4 and abs(f.mean()) < 5e-4


def test_hidden_states():
    h = bf16_bits_to_f32(make_hidden(10, 4096, 1))
    assert h.shape == (10, 4096)
    assert abs(h.std() - 1.0) < 0.02
    assert np.array_equal(make_hidden(10, 4096, 1), make_hidden(10, 4096, 1))


def test_ranking_is_a_permutation_sorted_by_count_then_id():
    r, counts = zipf_ranking(8192, 1.1, 10**6, 0)
    assert r.dtype == np.int32 and r.shape == (8192,)
    assert np.array_equal(np.sort(r), np.arange(8192))
    assert counts.sum() == 10**6
    c = counts[r]
    assert np.all(np.diff(c) <= 0)
    same = np.diff(c) == 0
    assert same.any()                       # the tie rule is exercised
    assert np.all(np.diff(r)[same] > 0)     # equal counts: lower id first
    r2, _ = zipf_ranking(8192, 1.1, 10**6, 0)
    assert np.array_equal(r, r2)


def test_ranking_has_the_papers_long_tail():
    paper, zipf = _golden_long_tail()
    for V, n, s, mass in zipf:
        j = np.arange(1, V + 1, dtype=np.float64) ** (-s)
        closed = j[:n].sum() / j.sum()
        assert abs(closed - mass) < 1e-3
    # the Llama-3-shaped stand-in: top 25.5% of ids must carry ~ the paper's 95%
    V, n, s, mass = zipf[0]
    r, counts = zipf_ranking(V, s, 10**7, 1)
    head = counts[r[:n]].sum() / counts.sum()
    assert abs(head - mass) < 0.005
    assert abs(n / V - paper["paper_head_fraction"]) < 0.01
    assert abs(head - paper["paper_head_mass"]) < 0.02


def test_exact_case_is_exactly_representable():
    W_bits, H_bits, W_int, H_int = make_exact_case(32, 64, 3, 1)
    assert np.array_equal(bf16_bits_to_f32(W_bits), W_int.astype(np.float32))
    assert np.array_equal(bf16_bits_to_f32(H_bits), H_int.astype(np.float32))
    assert np.abs(H_int @ W_int.T).max() < 2 ** 24
