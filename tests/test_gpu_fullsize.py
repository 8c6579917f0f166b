"""GPU parity at the full benchmark shapes, in the launch configuration bench.py times.

The Llama-3-8B-shaped draft step (d=4096, V=128256, V_sub=32768, M=10, k=10) and its
vocabulary-subset sweep are compared with the oracle row by row (the oracle finishes
these in well under a second per call).  For the batched shapes (M=60, 64, 256) the GPU
computes every row and a seeded sample of rows is checked against the oracle: rows of H
are independent, so the oracle run on the sampled rows alone is exact for them.
"""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr
from parity_utils import bits_of, check_topk_against_oracle, to_dev_bf16, to_dev_i32
from synth import CONFIGS, SWEEP_V_SUB, make_hidden, make_weights, zipf_ranking

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def llama():
    c = CONFIGS["llama3_8b"]
    _say("generating", c.name)
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(c.M, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    return c, W, H, r, to_dev_bf16(W), to_dev_bf16(H), to_dev_i32(r)


def test_llama3_8b_gather_bit_exact(llama):
    c, W, H, r, W_d, H_d, r_d = llama
    _say("full-size gather")
    W_g, idx_g = fr.fr_build_subset(W_d, r_d, c.V_sub)
    torch.cuda.synchronize()
    idx = idx_g.cpu().numpy()
    assert np.array_equal(idx, r[:c.V_sub])
    got = bits_of(W_g)
    # all 32768 rows, 8 KiB each, against numpy's gather (the library form of Eq. 3)
    assert np.array_equal(got, W[r[:c.V_sub]])


@pytest.mark.parametrize("V_sub", SWEEP_V_SUB)
def test_llama3_8b_sweep_matches_oracle(llama, V_sub):
    c, W, H, r, W_d, H_d, r_d = llama
    _say("full-size draft, V_sub =", V_sub)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, c.k, want_logits=True)
    W_g, idx_g = fr.fr_build_subset(W_d, r_d, V_sub)
    ws = fr.new_workspace(c.M, c.d, c.V, c.k)
    ids_g, lp_g = fr.fr_draft_topk(H_d, W_g, idx_g, c.k, ws)
    torch.cuda.synchronize()
    frac = check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
    _say("  rows identical to the oracle:", frac)
    # the logits themselves, all M x V_sub of them
    z_g = fr.fr_draft_logits(H_d, W_g).cpu().numpy()
    err = float(np.max(np.abs(z_g - z_o)))
    _say("  max abs logit error:", err)
    assert err <= 1e-2 and err < 1e-4


def test_llama3_8b_full_topk_matches_oracle(llama):
    c, W, H, r, W_d, H_d, r_d = llama
    _say("full-size full-vocabulary head")
    ids_o, lp_o, z_o = oracle.full_topk(H, W, c.k, want_logits=True)
    ws = fr.new_workspace(c.M, c.d, c.V, c.k)
    ids_g, lp_g = fr.fr_full_topk(H_d, W_d, c.k, ws)
    torch.cuda.synchronize()
    frac = check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, None, ids_o, lp_o)
    _say("  rows identical to the oracle:", frac)


def test_llama3_8b_subset_is_filtered_full_head(llama):
    # property that holds at any size: the subset's candidates are the full head's sorted
    # list restricted to V_high (near ties aside), and its logp is the full logp shifted
    # by the log of the subset's probability mass
    c, W, H, r, W_d, H_d, r_d = llama
    W_g, idx_g = fr.fr_build_subset(W_d, r_d, c.V_sub)
    ws = fr.new_workspace(c.M, c.d, c.V, 64)
    ids_s, lp_s = fr.fr_draft_topk(H_d, W_g, idx_g, c.k, ws)
    ids_f, lp_f = fr.fr_full_topk(H_d, W_d, 64, ws)
    torch.cuda.synchronize()
    ids_s, lp_s, ids_f, lp_f = (t.cpu().numpy() for t in (ids_s, lp_s, ids_f, lp_f))
    in_subset = set(int(t) for t in r[:c.V_sub])
    for m in range(c.M):
        full_lp = {int(t): float(v) for t, v in zip(ids_f[m], lp_f[m])}
        # every subset member among the full head's best 64 that beats the subset's k-th
        # candidate must have been returned by the subset head
        kth = float(lp_s[m, -1])
        shifts = [float(lp_s[m, j]) - full_lp[int(t)] for j, t in enumerate(ids_s[m]) if int(t) in full_lp]
        assert len(shifts) >= 3
        assert min(shifts) > 0 and max(shifts) - min(shifts) < 2e-2     # one constant: -log(mass)
        shift = float(np.mean(shifts))
        for t, v in full_lp.items():
            if t in in_subset and v + shift > kth + 2e-2:
                assert t in set(int(x) for x in ids_s[m]), (m, t)


def _sampled_rows_check(cfg_name, rows, full):
    c = CONFIGS[cfg_name]
    _say("generating", c.name)
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(c.M, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    W_d, H_d = to_dev_bf16(W), to_dev_bf16(H)
    sample = np.sort(np.random.default_rng(c.index).choice(c.M, size=rows, replace=False))
    ws = fr.new_workspace(c.M, c.d, c.V, c.k)
    if full:
        ids_g, lp_g = fr.fr_full_topk(H_d, W_d, c.k, ws)
        torch.cuda.synchronize()
        ids_o, lp_o, z_o = oracle.full_topk(H[sample], W, c.k, want_logits=True)
        idx_o = None
    else:
        W_g, idx_g = fr.fr_build_subset(W_d, to_dev_i32(r), c.V_sub)
        ids_g, lp_g = fr.fr_draft_topk(H_d, W_g, idx_g, c.k, ws)
        torch.cuda.synchronize()
        W_o, idx_o = oracle.build_subset(W, r, c.V_sub)
        assert np.array_equal(idx_g.cpu().numpy(), idx_o)
        ids_o, lp_o, z_o = oracle.draft_topk(H[sample], W_o, idx_o, c.k, want_logits=True)
    frac = check_topk_against_oracle(ids_g.cpu().numpy()[sample], lp_g.cpu().numpy()[sample], z_o, idx_o,
                                     ids_o, lp_o)
    _say("  sampled rows identical to the oracle:", frac)


def test_qwen25_7b_shape_sampled_rows():
    _sampled_rows_check("qwen25_7b", rows=12, full=False)


def test_batched256_shape_sampled_rows():
    _sampled_rows_check("batched256", rows=12, full=False)


def test_every_build_of_the_chunked_kernel_at_full_size():
    # the batched configuration's weights and ranking with the first M of its 256 rows of H: one
    # M per build of the chunked kernel (16, 32, 48, 64, 96 and 128 rows; the 8-wavefront skinny
    # kernel stops at 12 rows for d = 4096)
    c = CONFIGS["batched256"]
    _say("generating", c.name)
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(c.M, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), c.V_sub)
    W_o, idx_o = oracle.build_subset(W, r, c.V_sub)
    assert np.array_equal(idx_g.cpu().numpy(), idx_o)
    ws = fr.new_workspace(128, c.d, c.V_sub, c.k)
    for M in (14, 30, 48, 64, 96, 128):
        _say("  rows of H:", M)
        ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H[:M]), W_g, idx_g, c.k, ws)
        torch.cuda.synchronize()
        sample = np.sort(np.random.default_rng(M).choice(M, size=4, replace=False))
        ids_o, lp_o, z_o = oracle.draft_topk(H[sample], W_o, idx_o, c.k, want_logits=True)
        check_topk_against_oracle(ids_g.cpu().numpy()[sample], lp_g.cpu().numpy()[sample], z_o, idx_o,
                                  ids_o, lp_o)


def test_full_vocab_m64_sampled_rows():
    # the uncompressed head at M=64, the comparison point of the batched configuration
    c = CONFIGS["batched256"]
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(64, c.d, c.index)
    W_d, H_d = to_dev_bf16(W), to_dev_bf16(H)
    ws = fr.new_workspace(64, c.d, c.V, c.k)
    ids_g, lp_g = fr.fr_full_topk(H_d, W_d, c.k, ws)
    torch.cuda.synchronize()
    sample = np.array([0, 7, 21, 33, 48, 63])
    ids_o, lp_o, z_o = oracle.full_topk(H[sample], W, c.k, want_logits=True)
    frac = check_topk_against_oracle(ids_g.cpu().numpy()[sample], lp_g.cpu().numpy()[sample], z_o, None,
                                     ids_o, lp_o)
    _say("  sampled rows identical to the oracle:", frac)
