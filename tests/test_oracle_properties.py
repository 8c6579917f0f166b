"""Property tests of the CPU oracle on small random shapes (hypothesis): the invariants that
Eq. 2-4 fix, for any shape and any ranking, not just the hand-picked cases of the pins."""

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from synth import bf16_bits_to_f32, f32_to_bf16_bits


@st.composite
def head_case(draw):
    V = draw(st.integers(2, 48))
    d = draw(st.sampled_from([8, 16, 24]))
    M = draw(st.integers(1, 4))
    V_sub = draw(st.integers(1, V))
    k = draw(st.integers(1, V_sub))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    quantised = draw(st.booleans())          # small integers: exact arithmetic and many ties
    g = np.random.default_rng(seed)
    if quantised:
        W = g.integers(-2, 3, size=(V, d)).astype(np.float32)
        H = g.integers(-2, 3, size=(M, d)).astype(np.float32)
    else:
        W = (g.standard_normal((V, d)) * 0.5).astype(np.float32)
        H = g.standard_normal((M, d)).astype(np.float32)
    return f32_to_bf16_bits(W), f32_to_bf16_bits(H), g.permutation(V).astype(np.int32), V_sub, k


@settings(max_examples=150, deadline=None)
@given(head_case())
def test_subset_head_is_the_filtered_and_renormalised_full_head(case):
    W, H, r, V_sub, k = case
    V = W.shape[0]
    W_sub, idx = oracle.build_subset(W, r, V_sub)
    ids_s, lp_s, z_s = oracle.draft_topk(H, W_sub, idx, k, want_logits=True)
    ids_f, lp_f, z_f = oracle.full_topk(H, W, V, want_logits=True)     # the full head, fully sorted
    # restriction: the subset's logits are the full logits at the chosen ids, bit for bit
    assert np.array_equal(z_s, z_f[:, r[:V_sub]])
    members = set(int(t) for t in r[:V_sub])
    for m in range(H.shape[0]):
        # filter: the subset's candidates are the full head's sorted list restricted to V_high
        want = [int(t) for t in ids_f[m] if int(t) in members][:k]
        assert [int(t) for t in ids_s[m]] == want
        # Eq. 4 normalises over the subset only: probabilities of all members sum to one, and
        # logp_sub(t) = logp_full(t) - log(mass of the subset under the full distribution)
        z64 = z_s[m].astype(np.float64)
        logZ = np.log(np.sum(np.exp(z64 - z64.max()))) + z64.max()
        full = {int(t): float(v) for t, v in zip(ids_f[m], lp_f[m])}
        mass = np.log(sum(np.exp(full[t]) for t in members))
        for j, t in enumerate(ids_s[m]):
            pos = int(np.nonzero(idx == t)[0][0])
            assert abs(float(lp_s[m, j]) - (z64[pos] - logZ)) < 1e-5
            assert abs(float(lp_s[m, j]) - (full[int(t)] - mass)) < 1e-4
        # order: logit descending, equal logits by lower full-vocabulary id
        keys = [(-float(z_s[m, int(np.nonzero(idx == t)[0][0])]), int(t)) for t in ids_s[m]]
        assert keys == sorted(keys)


@settings(max_examples=60, deadline=None)
@given(head_case())
def test_order_inside_v_high_does_not_matter(case):
    W, H, r, V_sub, k = case
    W_a, idx_a = oracle.build_subset(W, r, V_sub)
    shuffled = r.copy()
    shuffled[:V_sub] = shuffled[:V_sub][::-1]
    W_b, idx_b = oracle.build_subset(W, shuffled, V_sub)
    ids_a, lp_a = oracle.draft_topk(H, W_a, idx_a, k)
    ids_b, lp_b = oracle.draft_topk(H, W_b, idx_b, k)
    assert np.array_equal(ids_a, ids_b)
    assert np.max(np.abs(lp_a - lp_b)) < 1e-5      # the normaliser is summed in another order


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 40), st.integers(1, 3000), st.integers(0, 2 ** 31 - 1))
def test_counting_and_ranking_follow_numpy(V, n, seed):
    g = np.random.default_rng(seed)
    tokens = g.integers(-2, V + 2, size=n).astype(np.int32)
    counts, bad = oracle.count_tokens(tokens, V)
    ok = tokens[(tokens >= 0) & (tokens < V)]
    assert np.array_equal(counts, np.bincount(ok, minlength=V)) and bad == n - ok.size
    ranked = oracle.rank_tokens(counts)
    assert np.array_equal(ranked, np.lexsort((np.arange(V), -counts)))
