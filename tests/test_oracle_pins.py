"""Pins of the CPU oracle against things other than itself.

The paper prints no numbers for the draft-head path, so the oracle is pinned
by what Eq. 2-4 and the mathematics fix: integer-exact inputs checked with
int64 arithmetic, closed forms (uniform rows), library routines on the special
case V_sub = V (matmul + log_softmax + topk of torch on the CPU), brute force
on tiny inputs, and the invariants that relate the subset head (Eq. 4) to the
full head (Eq. 2).  Each test is chosen so that one plausible mistake (a
transposed operand, a dropped remap, normalising over the wrong set, a wrong
tie rule) fails it.
"""

import itertools
import math

import numpy as np
import pytest
import torch

import oracle
from synth import bf16_bits_to_f32, f32_to_bf16_bits, make_exact_case, make_hidden, make_weights


def _rand_case(V, d, M, seed, w_std=0.02):
    g = np.random.default_rng(seed)
    W = f32_to_bf16_bits((g.standard_normal((V, d)) * w_std).astype(np.float32))
    H = f32_to_bf16_bits(g.standard_normal((M, d)).astype(np.float32))
    r = g.permutation(V).astype(np.int32)
    return W, H, r


# ----------------------------------------------------------------- Eq. 3 ---

def test_gather_identity_is_a_copy():
    W, _, _ = _rand_case(97, 24, 1, 1)
    W_sub, idx = oracle.build_subset(W, np.arange(97, dtype=np.int32), 97)
    assert np.array_equal(W_sub, W)
    assert np.array_equal(idx, np.arange(97))


def test_gather_row_i_is_row_r_i():
    W, _, r = _rand_case(211, 40, 1, 2)
    V_sub = 50
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    assert W_sub.shape == (V_sub, 40)
    for i in range(V_sub):
        assert np.array_equal(W_sub[i], W[r[i]])
    assert np.array_equal(idx, r[:V_sub])
    # numpy fancy indexing is the library form of Eq. 3
    assert np.array_equal(W_sub, W[r[:V_sub]])


def test_gather_rejects_bad_ids():
    W, _, r = _rand_case(16, 8, 1, 3)
    bad = r.copy()
    bad[3] = 16
    with pytest.raises(oracle.OracleError):
        oracle.build_subset(W, bad, 8)
    bad[3] = -1
    with pytest.raises(oracle.OracleError):
        oracle.build_subset(W, bad, 8)
    with pytest.raises(oracle.OracleError):
        oracle.build_subset(W, r, 17)


# ---------------------------------------------------------------- logits ---

def test_logits_exact_integer_inputs_match_int64_matmul():
    # Every partial sum is an integer below 2^24: the fp32 result must equal the
    # int64 product bit for bit.  A transposed or mis-indexed operand fails here.
    W_bits, H_bits, W_int, H_int = make_exact_case(V=130, d=96, M=5, seed=0)
    z = oracle.logits_f32(H_bits, W_bits)
    exact = H_int @ W_int.T
    assert z.shape == (5, 130)
    assert np.array_equal(z.astype(np.int64), exact)
    assert np.array_equal(z, exact.astype(np.float32))
    z64 = oracle.logits_f64(H_bits, W_bits)
    assert np.array_equal(z64, exact.astype(np.float64))


def test_logits_one_hot_h_reads_a_column():
    W, _, _ = _rand_case(64, 32, 1, 4)
    for j in (0, 7, 31):
        h = np.zeros((1, 32), dtype=np.float32)
        h[0, j] = 1.0
        z = oracle.logits_f32(f32_to_bf16_bits(h), W)
        assert np.array_equal(z[0], bf16_bits_to_f32(W[:, j]))


def test_logits_match_library_matmul_and_fp64():
    W, H, _ = _rand_case(300, 512, 7, 5)
    z = oracle.logits_f32(H, W)
    Wf = torch.from_numpy(bf16_bits_to_f32(W))
    Hf = torch.from_numpy(bf16_bits_to_f32(H))
    z_lib = (Hf.double() @ Wf.double().T).numpy()
    assert np.max(np.abs(z - z_lib)) < 1e-4
    z64 = oracle.logits_f64(H, W)
    assert np.max(np.abs(z64 - z_lib)) < 1e-10
    assert np.max(np.abs(z - z64)) < 1e-4


def test_logits_restriction_invariant_is_bit_exact():
    # Eq. 4 is Eq. 2 on fewer rows: z_sub[m, i] == z_full[m, r[i]] exactly.
    W, H, r = _rand_case(257, 128, 3, 6)
    V_sub = 100
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    z_full = oracle.logits_f32(H, W)
    z_sub = oracle.logits_f32(H, W_sub)
    assert np.array_equal(z_sub, z_full[:, idx])


# ----------------------------------------------------------- log-softmax ---

def test_log_softmax_normalises_and_matches_library():
    g = np.random.default_rng(7)
    z = (g.standard_normal((6, 1000)) * 3).astype(np.float32)
    logp, logZ = oracle.log_softmax(z)
    assert np.allclose(np.exp(logp.astype(np.float64)).sum(axis=1), 1.0, atol=1e-5)
    ref = torch.log_softmax(torch.from_numpy(z).double(), dim=1).numpy()
    assert np.max(np.abs(logp - ref)) < 1e-5
    ref_lz = torch.logsumexp(torch.from_numpy(z).double(), dim=1).numpy()
    assert np.max(np.abs(logZ - ref_lz)) < 1e-9


def test_log_softmax_shift_invariance():
    g = np.random.default_rng(8)
    z = g.standard_normal((2, 64)).astype(np.float32)
    z2 = z + np.float32(8.0)   # exactly representable shift at this magnitude range
    lp1, _ = oracle.log_softmax(z)
    lp2, _ = oracle.log_softmax(z2)
    assert np.max(np.abs(lp1 - lp2)) < 2e-6


def test_uniform_rows_closed_form():
    # All rows of W equal  =>  uniform distribution over the subset: logp = -log(V_sub),
    # and the tie rule must return the k lowest full-vocabulary ids of the subset.
    V, d, V_sub, k = 50, 16, 20, 5
    row = f32_to_bf16_bits(np.linspace(-1, 1, d).astype(np.float32))
    W = np.tile(row, (V, 1))
    H = f32_to_bf16_bits(np.ones((2, d), dtype=np.float32))
    r = np.random.default_rng(9).permutation(V).astype(np.int32)
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    ids, logp = oracle.draft_topk(H, W_sub, idx, k)
    assert np.allclose(logp, -math.log(V_sub), atol=1e-6)
    expect = np.sort(r[:V_sub])[:k]
    assert np.array_equal(ids[0], expect) and np.array_equal(ids[1], expect)


def test_zero_hidden_state_closed_form():
    W, _, r = _rand_case(40, 8, 1, 10)
    H = np.zeros((1, 8), dtype=np.uint16)
    ids, logp = oracle.full_topk(H, W, 3)
    assert np.array_equal(ids[0], [0, 1, 2])
    assert np.allclose(logp, -math.log(40), atol=1e-6)


def test_subset_renormalisation_identity():
    # logp_sub(t) = logp_full(t) - log sum_{u in V_high} p_full(u)
    W, H, r = _rand_case(400, 64, 4, 11, w_std=0.3)
    V_sub = 120
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    z_full = oracle.logits_f32(H, W)
    lp_full, _ = oracle.log_softmax(z_full)
    z_sub = oracle.logits_f32(H, W_sub)
    lp_sub, _ = oracle.log_softmax(z_sub)
    mass = np.log(np.exp(lp_full[:, idx].astype(np.float64)).sum(axis=1))
    assert np.max(np.abs(lp_sub - (lp_full[:, idx] - mass[:, None]))) < 1e-5
    # and a larger subset can only lower a fixed token's log-probability
    W_sub2, idx2 = oracle.build_subset(W, r, 300)
    lp_sub2, _ = oracle.log_softmax(oracle.logits_f32(H, W_sub2))
    assert np.all(lp_sub2[:, :V_sub] <= lp_sub + 1e-6)


# ------------------------------------------------------------------ top-k ---

def _brute_topk(z_row, ids, k):
    """Exhaustive: the k-subset, in an order, that is lexicographically best."""
    n = len(z_row)
    best = None
    for combo in itertools.permutations(range(n), k):
        key = tuple((-float(z_row[i]), int(ids[i])) for i in combo)
        if best is None or key < best[0]:
            best = (key, combo)
    return [int(ids[i]) for i in best[1]]


def test_topk_brute_force_tiny():
    g = np.random.default_rng(12)
    for trial in range(6):
        n = 6
        z = g.integers(-2, 3, size=(1, n)).astype(np.float32)   # many exact ties
        ids_map = g.permutation(50)[:n].astype(np.int32)
        for k in range(1, 5):
            got, _ = oracle.topk(z, ids_map, k)
            assert got[0].tolist() == _brute_topk(z[0], ids_map, k), (trial, k)


def test_topk_matches_lexsort_and_full_sort():
    g = np.random.default_rng(13)
    z = np.round(g.standard_normal((3, 500)) * 4).astype(np.float32) / 4   # ties
    ids_map = g.permutation(5000)[:500].astype(np.int32)
    for k in (1, 10, 64, 500):
        got, pos = oracle.topk(z, ids_map, k)
        for m in range(3):
            order = np.lexsort((ids_map, -z[m]))[:k]
            assert np.array_equal(got[m], ids_map[order])
            assert np.array_equal(pos[m], order)


def test_topk_tie_rule_uses_full_vocab_id_not_subset_position():
    # Two identical W rows; the one with the LOWER full id sits LATER in rank order.
    d = 8
    W = f32_to_bf16_bits(np.random.default_rng(14).standard_normal((10, d)).astype(np.float32))
    W[2] = W[7]
    H = f32_to_bf16_bits(bf16_bits_to_f32(W[7:8]) * 4)   # makes rows 2 and 7 the top pair
    r = np.array([7, 5, 2, 0, 1, 3, 4, 6, 8, 9], dtype=np.int32)   # 7 ranked before 2
    W_sub, idx = oracle.build_subset(W, r, 6)
    ids, logp = oracle.draft_topk(H, W_sub, idx, 2)
    assert ids[0].tolist() == [2, 7]
    assert logp[0, 0] == logp[0, 1]


def test_subset_topk_is_filtered_full_topk():
    W, H, r = _rand_case(600, 64, 5, 15, w_std=0.2)
    V_sub, k = 150, 12
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    ids_sub, _ = oracle.draft_topk(H, W_sub, idx, k)
    ids_full, _ = oracle.full_topk(H, W, 600)   # the whole sorted list
    member = np.zeros(600, dtype=bool)
    member[idx] = True
    for m in range(5):
        filtered = [t for t in ids_full[m] if member[t]][:k]
        assert ids_sub[m].tolist() == filtered


def test_subset_order_within_v_high_does_not_matter():
    W, H, r = _rand_case(300, 32, 3, 16, w_std=0.2)
    V_sub, k = 90, 7
    r2 = r.copy()
    r2[:V_sub] = np.random.default_rng(17).permutation(r[:V_sub])
    a = oracle.draft_topk(H, *oracle.build_subset(W, r, V_sub), k)
    b = oracle.draft_topk(H, *oracle.build_subset(W, r2, V_sub), k)
    assert np.array_equal(a[0], b[0])
    assert np.max(np.abs(a[1] - b[1])) < 1e-6


# ------------------------------------------------------------ whole path ---

def test_remap_ids_are_distinct_members_of_v_high():
    W, H, r = _rand_case(500, 48, 6, 18)
    V_sub, k = 128, 10
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    ids, logp = oracle.draft_topk(H, W_sub, idx, k)
    allowed = set(r[:V_sub].tolist())
    for m in range(6):
        assert len(set(ids[m].tolist())) == k
        assert set(ids[m].tolist()) <= allowed
        assert np.all(np.diff(logp[m]) <= 0)


def test_v_sub_equal_v_is_the_full_head_and_the_library_routine():
    W, H, _ = _rand_case(777, 256, 4, 19, w_std=0.05)
    V, k = 777, 9
    W_sub, idx = oracle.build_subset(W, np.arange(V, dtype=np.int32), V)
    a_ids, a_lp = oracle.draft_topk(H, W_sub, idx, k)
    b_ids, b_lp = oracle.full_topk(H, W, k)
    assert np.array_equal(a_ids, b_ids) and np.array_equal(a_lp, b_lp)
    # textbook routine: matmul + log_softmax + topk
    Wf = torch.from_numpy(bf16_bits_to_f32(W)).double()
    Hf = torch.from_numpy(bf16_bits_to_f32(H)).double()
    lp = torch.log_softmax(Hf @ Wf.T, dim=1)
    val, ind = torch.topk(lp, k, dim=1)
    assert np.array_equal(b_ids, ind.numpy().astype(np.int32))   # no ties in random data
    assert np.max(np.abs(b_lp - val.numpy())) < 1e-4


def test_returned_logits_are_the_logits():
    W, H, r = _rand_case(128, 64, 2, 20)
    W_sub, idx = oracle.build_subset(W, r, 64)
    ids, logp, z = oracle.draft_topk(H, W_sub, idx, 3, want_logits=True)
    assert np.array_equal(z, oracle.logits_f32(H, W_sub))
    lp_all, _ = oracle.log_softmax(z)
    pos = {int(t): i for i, t in enumerate(idx)}
    for m in range(2):
        for j in range(3):
            assert logp[m, j] == lp_all[m, pos[int(ids[m, j])]]


def test_generated_workload_tiny_config_runs():
    W = make_weights(512, 64, 0)
    H = make_hidden(3, 64, 0)
    ids, logp = oracle.full_topk(H, W, 4)
    assert ids.shape == (3, 4) and np.all(np.isfinite(logp))
