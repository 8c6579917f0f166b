"""GPU parity of the draft-step glue (beam expansion, draft-tree selection) against the CPU
oracle: everything here is integer work or a single fp32 addition, so every output is
compared bit for bit."""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


@pytest.mark.parametrize("seed,M,k,width,off", [(0, 1, 10, 10, 0), (1, 10, 10, 10, 10), (2, 10, 10, 100, 110),
                                                (3, 16, 16, 7, 3), (4, 60, 10, 60, 0), (5, 64, 64, 333, 17),
                                                (6, 1, 1, 1, 0)])
def test_beam_expand_matches_oracle_bit_for_bit(seed, M, k, width, off):
    _say("beam expand", seed, M, k, width, off)
    rng = np.random.default_rng([20250214, 91, seed])
    quantised = seed % 2 == 0          # exactly equal cumulative scores: the tie rule decides
    logp = (-rng.integers(0, 12, size=(M, k)) / 4 if quantised else -rng.exponential(2.0, size=(M, k)))
    logp = logp.astype(np.float32)
    if seed == 3:
        logp[:, -2:] = -np.inf         # rows with fewer than k real candidates
    tok = rng.integers(0, 128256, size=(M, k)).astype(np.int32)
    node_score = (-rng.integers(0, 8, size=M) / 2).astype(np.float32)
    node_hist = rng.integers(-1, max(off, 1), size=M).astype(np.int32)
    n = off + M * k
    hs_o, ht_o, hp_o = np.full(n, 7.0, np.float32), np.full(n, 7, np.int32), np.full(n, 7, np.int32)
    want = oracle.beam_expand(logp, tok, node_score, node_hist, width, hs_o, ht_o, hp_o, off)
    hs_g, ht_g, hp_g = _dev(np.full(n, 7.0, np.float32)), _dev(np.full(n, 7, np.int32)), _dev(np.full(n, 7, np.int32))
    got = fr.fr_beam_expand(_dev(logp), _dev(tok), _dev(node_score), _dev(node_hist), width, hs_g, ht_g, hp_g, off)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(hs_g.cpu().numpy()), _bits(hs_o))
    assert np.array_equal(ht_g.cpu().numpy(), ht_o) and np.array_equal(hp_g.cpu().numpy(), hp_o)
    assert np.array_equal(_bits(got[0].cpu().numpy()), _bits(want[0]))
    assert np.array_equal(got[1].cpu().numpy(), want[1]) and np.array_equal(got[2].cpu().numpy(), want[2])


def _random_history(rng, n, quantised):
    parent = np.empty(n, dtype=np.int32)
    score = np.empty(n, dtype=np.float32)
    for i in range(n):
        parent[i] = -1 if i < min(n, 10) else int(rng.integers(-1, i))
        step = -float(rng.integers(0, 6)) / 4 if quantised else -float(rng.exponential(1.0))
        score[i] = np.float32((0.0 if parent[i] < 0 else score[parent[i]]) + np.float32(step))
    return score, rng.integers(0, 128256, size=n).astype(np.int32), parent


# (from 2K-and-more groups of at least two entries on, the selection goes through a bound and ranks
# only the entries above it: 510/60, 610/60, 256/64 (exactly two per group), 300/60, 3000/300, 4096/...)
@pytest.mark.parametrize("seed,n,K", [(0, 40, 12), (1, 610, 60), (2, 610, 60), (3, 100, 100), (4, 1, 1),
                                      (5, 4096, 128), (6, 1500, 1024), (7, 33, 32), (8, 510, 60), (9, 256, 64),
                                      (10, 300, 60), (11, 3000, 300), (12, 4096, 512), (13, 4095, 1),
                                      (14, 255, 64), (16, 4096, 33)])
def test_tree_select_matches_oracle_bit_for_bit(seed, n, K):
    _say("tree select", seed, n, K)
    rng = np.random.default_rng([20250214, 92, seed])
    score, token, parent = _random_history(rng, n, quantised=seed % 2 == 0)
    want = oracle.tree_select(score, token, parent, K)
    got = fr.fr_tree_select(_dev(score), _dev(token), _dev(parent), n, K)
    torch.cuda.synchronize()
    for g, w, name in zip(got, want, ("sel_index", "sel_token", "sel_parent", "sel_depth", "tree_mask")):
        assert np.array_equal(g.cpu().numpy(), w), name


def test_six_step_draft_with_the_lm_head_in_the_loop():
    # the whole draft phase at the paper's setting (depth 6, 60 draft tokens; beam width 10 is
    # this build's reading): fr_draft_topk -> fr_beam_expand per step, then fr_tree_select.
    # The hidden state of a node is synthetic: a seeded function of (step, node).
    from parity_utils import to_dev_bf16, to_dev_i32
    from synth import make_hidden, make_weights, zipf_ranking
    _say("six-step draft")
    d, V, V_sub, k, width, depth, K = 256, 8192, 2048, 10, 10, 6, 60
    W = make_weights(V, d, 0)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 0)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(width, d, V, k)
    cap = k + (depth - 1) * width * k
    hs_o, ht_o, hp_o = np.zeros(cap, np.float32), np.zeros(cap, np.int32), np.zeros(cap, np.int32)
    hs_g, ht_g, hp_g = _dev(hs_o), _dev(ht_o), _dev(hp_o)
    ns_o, nh_o = np.zeros(1, np.float32), np.full(1, -1, np.int32)
    ns_g, nh_g = _dev(ns_o), _dev(nh_o)
    off = 0
    for step in range(depth):
        M = len(ns_o)
        H = make_hidden(M, d, 100 + step)
        ids_o, lp_o = oracle.draft_topk(H, W_o, idx_o, k)
        ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws)
        torch.cuda.synchronize()
        assert np.array_equal(ids_g.cpu().numpy(), ids_o)
        # the glue is compared on identical inputs: feed both sides the oracle's log-probabilities
        ns_o, _, nh_o = oracle.beam_expand(lp_o, ids_o, ns_o, nh_o, min(width, M * k), hs_o, ht_o, hp_o, off)
        ns_g, _, nh_g = fr.fr_beam_expand(_dev(lp_o), ids_g, ns_g, nh_g, min(width, M * k), hs_g, ht_g, hp_g, off)
        off += M * k
    assert off == cap
    want = oracle.tree_select(hs_o, ht_o, hp_o, K)
    got = fr.fr_tree_select(hs_g, ht_g, hp_g, off, K)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(hs_g.cpu().numpy()), _bits(hs_o))
    for g, w in zip(got, want):
        assert np.array_equal(g.cpu().numpy(), w)
    assert (want[2] != -2).all()            # every selected entry has its parent selected
    assert int(want[3].max()) <= depth - 1


@pytest.mark.parametrize("M,k,width,V_sub,off", [(1, 10, 10, 2048, 0), (10, 10, 10, 2048, 10), (16, 16, 50, 3000, 7),
                                                 (10, 10, 100, 300, 0), (4, 4, 3, 64, 5),
                                                 (10, 20, 10, 2048, 0), (20, 10, 10, 2048, 0)])
def test_fused_draft_step_equals_the_two_calls(M, k, width, V_sub, off):
    # fr_draft_step = fr_draft_topk + fr_beam_expand; for M <= 16, k <= 16 inside one launch.
    # The fused path sees the same log-probabilities, so everything must agree bit for bit; the
    # two calls themselves are checked against the oracle elsewhere.
    from parity_utils import to_dev_bf16, to_dev_i32
    from synth import make_hidden, make_weights, zipf_ranking
    _say("fused draft step", M, k, width, V_sub, off)
    d, V = 256, 8192
    W = make_weights(V, d, 2)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 2)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V, k)
    rng = np.random.default_rng([20250214, 101, M, k])
    node_score = _dev((-rng.integers(0, 8, size=M) / 2).astype(np.float32))
    node_hist = _dev(rng.integers(-1, max(off, 1), size=M).astype(np.int32))
    n = off + M * k
    for rep in range(2):       # twice on one workspace: the hand-over records must be empty again
        H = to_dev_bf16(make_hidden(M, d, 200 + rep))
        hist_a = [_dev(np.full(n, 7.0, np.float32)), _dev(np.full(n, 7, np.int32)), _dev(np.full(n, 7, np.int32))]
        hist_b = [t.clone() for t in hist_a]
        ids_a, lp_a = fr.fr_draft_topk(H, W_g, idx_g, k, ws)
        nxt_a = fr.fr_beam_expand(lp_a, ids_a, node_score, node_hist, width, *hist_a, off)
        ids_b, lp_b, *nxt_b = fr.fr_draft_step(H, W_g, idx_g, k, node_score, node_hist, width, *hist_b, off, ws)
        torch.cuda.synchronize()
        assert np.array_equal(ids_b.cpu().numpy(), ids_a.cpu().numpy())
        assert np.array_equal(_bits(lp_b.cpu().numpy()), _bits(lp_a.cpu().numpy()))
        for x, y in zip(hist_a + list(nxt_a), hist_b + list(nxt_b)):
            xa, ya = x.cpu().numpy(), y.cpu().numpy()
            assert np.array_equal(xa.view(np.uint32), ya.view(np.uint32))
        step_region = ws[512 + (16 * 16 + 16) * 512 * 8:][:16 * 16 * 8].cpu().numpy()
        assert (step_region == 0xFF).all()
    assert fr.fr_workspace_check(ws) is False


def test_six_fused_steps_equal_six_unfused_steps():
    from parity_utils import to_dev_bf16, to_dev_i32
    from synth import make_hidden, make_weights, zipf_ranking
    d, V, V_sub, k, width, depth, K = 256, 8192, 2048, 10, 10, 6, 60
    W = make_weights(V, d, 0)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 0)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(width, d, V, k)
    cap = k + (depth - 1) * width * k
    out = []
    for fused in (False, True):
        hist = [torch.zeros(cap, dtype=torch.float32, device="cuda"), torch.zeros(cap, dtype=torch.int32, device="cuda"),
                torch.zeros(cap, dtype=torch.int32, device="cuda")]
        ns = torch.zeros(1, dtype=torch.float32, device="cuda")
        nh = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        off = 0
        for step in range(depth):
            M = ns.numel()
            H = to_dev_bf16(make_hidden(M, d, 100 + step))
            if fused:
                _, _, ns, _, nh = fr.fr_draft_step(H, W_g, idx_g, k, ns, nh, min(width, M * k), *hist, off, ws)
            else:
                ids, lp = fr.fr_draft_topk(H, W_g, idx_g, k, ws)
                ns, _, nh = fr.fr_beam_expand(lp, ids, ns, nh, min(width, M * k), *hist, off)
            off += M * k
        sel = fr.fr_tree_select(*hist, off, K)
        torch.cuda.synchronize()
        out.append([t.cpu().numpy() for t in hist + list(sel)])
    for a, b in zip(*out):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


@pytest.mark.parametrize("M,k,width,V_sub,off,d", [(1, 10, 10, 2048, 0, 256), (10, 10, 10, 2048, 10, 256),
                                                   (16, 16, 50, 3000, 7, 256), (10, 10, 10, 32768, 10, 4096),
                                                   (10, 20, 10, 2048, 0, 256), (20, 10, 10, 2048, 0, 256)])
def test_fused_draft_step_against_the_oracle(M, k, width, V_sub, off, d):
    # fr_draft_step against oracle.draft_topk followed by oracle.beam_expand, with nothing of
    # the library in between: tokens and parents bit for bit, scores inside the band of the
    # log-probabilities (the head's logp differs from the oracle's in the last bits, and the
    # cumulative score is one fp32 addition on top), next nodes equal except at near ties of
    # the oracle's own scores.  The last-but-two case is the benchmark's shape.
    from parity_utils import TIGHT_TOL, to_dev_bf16, to_dev_i32
    from synth import make_hidden, make_weights, zipf_ranking
    _say("fused draft step vs oracle", M, k, width, V_sub, off, d)
    V = 8192 if d == 256 else 40000
    W = make_weights(V, d, 3)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 3)
    H = make_hidden(M, d, 300 + M)
    rng = np.random.default_rng([20250214, 103, M, k])
    node_score = (-rng.integers(0, 8, size=M) / 2).astype(np.float32)
    node_hist = rng.integers(-1, max(off, 1), size=M).astype(np.int32)
    n = off + M * k
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
    hs_o, ht_o, hp_o = np.full(n, 7.0, np.float32), np.full(n, 7, np.int32), np.full(n, 7, np.int32)
    ns_o, nt_o, nh_o = oracle.beam_expand(lp_o, ids_o, node_score, node_hist, width, hs_o, ht_o, hp_o, off)

    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V, k)
    hist_g = [_dev(np.full(n, 7.0, np.float32)), _dev(np.full(n, 7, np.int32)), _dev(np.full(n, 7, np.int32))]
    ids_g, lp_g, ns_g, nt_g, nh_g = fr.fr_draft_step(to_dev_bf16(H), W_g, idx_g, k, _dev(node_score), _dev(node_hist),
                                                     width, *hist_g, off, ws)
    torch.cuda.synchronize()
    ids_g, lp_g = ids_g.cpu().numpy(), lp_g.cpu().numpy()
    hs_g, ht_g, hp_g = (t.cpu().numpy() for t in hist_g)
    ns_g, nt_g, nh_g = ns_g.cpu().numpy(), nt_g.cpu().numpy(), nh_g.cpu().numpy()
    # the head's own outputs
    same_ids = np.array_equal(ids_g, ids_o)
    if not same_ids:     # only a near tie of two logits may reorder candidates
        pos = {int(t): i for i, t in enumerate(idx_o)}
        for m, j in zip(*np.nonzero(ids_g != ids_o)):
            assert abs(z_o[m, pos[int(ids_g[m, j])]] - z_o[m, pos[int(ids_o[m, j])]]) < 1e-2
    assert np.array_equal(hs_g[:off], hs_o[:off]) and np.array_equal(ht_g[:off], ht_o[:off])   # untouched
    assert np.array_equal(hp_g, hp_o)                     # parents never depend on the arithmetic
    assert np.array_equal(ht_g[off:], ids_g.reshape(-1))  # the history holds what the head returned
    if same_ids:
        assert np.array_equal(ht_g, ht_o)
        assert float(np.max(np.abs(lp_g - lp_o))) < TIGHT_TOL
        assert float(np.max(np.abs(hs_g[off:] - hs_o[off:]))) < TIGHT_TOL
        # next nodes: the oracle's choice, except where its own scores at the two places tie closely
        for j in range(width):
            if nh_g[j] != nh_o[j]:
                assert abs(float(hs_o[nh_g[j]]) - float(hs_o[nh_o[j]])) < 2 * TIGHT_TOL, (j, nh_g[j], nh_o[j])
            assert nt_g[j] == ht_g[nh_g[j]] and ns_g[j] == hs_g[nh_g[j]]
        assert len(set(int(x) for x in nh_g)) == width
    # and the GPU's expansion is exactly the oracle's expansion of the GPU head's outputs
    hs2, ht2, hp2 = np.full(n, 7.0, np.float32), np.full(n, 7, np.int32), np.full(n, 7, np.int32)
    ns2, nt2, nh2 = oracle.beam_expand(lp_g, ids_g, node_score, node_hist, width, hs2, ht2, hp2, off)
    assert np.array_equal(_bits(hs_g), _bits(hs2)) and np.array_equal(ht_g, ht2)
    assert np.array_equal(_bits(ns_g), _bits(ns2)) and np.array_equal(nt_g, nt2) and np.array_equal(nh_g, nh2)
    assert fr.fr_workspace_check(ws) is False
