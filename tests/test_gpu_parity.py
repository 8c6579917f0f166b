"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Bar: gather / remap bit-exact; logits within 1e-2 max-abs; top-k ids
identical except at near ties of the oracle's own logits (< 1e-2); exact-arithmetic
inputs must agree with no exemption."""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr
from paper_2502_14856_amd.binding import Tuning
from parity_utils import (LOGIT_TOL, bits_of, check_topk_against_oracle, to_dev_bf16, to_dev_i32)
from synth import (CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_exact_case, make_hidden, make_weights,
                   zipf_ranking)

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _case(V, d, M, seed, w_std=0.05):
    g = np.random.default_rng([77, seed])
    W = f32_to_bf16_bits((g.standard_normal((V, d)) * w_std).astype(np.float32))
    H = f32_to_bf16_bits(g.standard_normal((M, d)).astype(np.float32))
    r = g.permutation(V).astype(np.int32)
    return W, H, r


def _sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------ Eq. 3 ---

@pytest.mark.parametrize("V,d,V_sub", [(8192, 256, 2048), (1000, 264, 1000), (777, 8, 1), (5000, 4096, 1234)])
def test_build_subset_bit_exact(V, d, V_sub):
    _say("gather", V, d, V_sub)
    W, _, r = _case(V, d, 1, 1)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub, dev_error_flag=flag)
    _sync()
    assert np.array_equal(bits_of(W_g), W_o)
    assert np.array_equal(idx_g.cpu().numpy(), idx_o)
    assert int(flag.item()) == 0


def test_build_subset_flags_bad_ids_without_faulting():
    _say("gather bad ids")
    W, _, r = _case(300, 64, 1, 2)
    bad = r.copy()
    bad[5] = 300
    bad[9] = -7
    W_sub = torch.zeros((20, 64), dtype=torch.bfloat16, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(bad), 20, W_sub=W_sub, dev_error_flag=flag)
    _sync()
    assert int(flag.item()) == 1
    got, idx = bits_of(W_g), idx_g.cpu().numpy()
    for i in range(20):
        if i in (5, 9):
            assert idx[i] == -1 and not got[i].any()      # row left untouched (zeros)
        else:
            assert idx[i] == bad[i] and np.array_equal(got[i], W[bad[i]])


def test_tiny_config_generated_ranking_gather():
    c = CONFIGS["tiny"]
    _say("gather tiny config")
    W = make_weights(c.V, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    W_o, idx_o = oracle.build_subset(W, r, c.V_sub)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), c.V_sub)
    _sync()
    assert np.array_equal(bits_of(W_g), W_o) and np.array_equal(idx_g.cpu().numpy(), idx_o)


# ----------------------------------------------------------------- logits ---

@pytest.mark.parametrize("M,d,V", [(1, 256, 2048), (4, 256, 2048), (10, 4096, 600), (16, 512, 1000),
                                   (7, 264, 333), (3, 8, 17), (10, 136, 129), (13, 1024, 4099)])
def test_logits_skinny_within_tolerance(M, d, V):
    _say("logits skinny", M, d, V)
    W, H, _ = _case(V, d, M, 3)
    z_o = oracle.logits_f32(H, W)
    z_g = fr.fr_draft_logits(to_dev_bf16(H), to_dev_bf16(W))
    _sync()
    err = np.max(np.abs(z_g.cpu().numpy() - z_o))
    _say("  max abs err", err)
    assert err <= LOGIT_TOL
    assert err < 1e-4      # what fp32 accumulation actually delivers at these sizes


@pytest.mark.parametrize("M,d,V", [(17, 256, 2048), (60, 512, 1000), (64, 4096, 300), (100, 264, 333),
                                   (256, 256, 513), (300, 128, 260), (45, 1024, 500), (90, 520, 333)])
def test_logits_matrix_core_within_tolerance(M, d, V):
    _say("logits mfma", M, d, V)
    W, H, _ = _case(V, d, M, 4)
    z_o = oracle.logits_f32(H, W)
    z_g = fr.fr_draft_logits(to_dev_bf16(H), to_dev_bf16(W))
    _sync()
    err = np.max(np.abs(z_g.cpu().numpy() - z_o))
    _say("  max abs err", err)
    assert err <= LOGIT_TOL
    assert err < 1e-4


@pytest.mark.parametrize("M", [1, 10, 16, 40, 256])
def test_logits_exact_inputs_bit_exact(M):
    _say("logits exact", M)
    W_bits, H_bits, W_int, H_int = make_exact_case(V=700, d=520, M=M, seed=M)
    exact = (H_int @ W_int.T).astype(np.float32)
    z_g = fr.fr_draft_logits(to_dev_bf16(H_bits), to_dev_bf16(W_bits))
    _sync()
    assert np.array_equal(z_g.cpu().numpy(), exact)


# ------------------------------------------------------------------ top-k ---

def _run_draft(W, H, r, V_sub, k, tuning=None, exact=False):
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
    M, d = H.shape
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V_sub, k)
    ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws, tuning=tuning)
    _sync()
    frac = check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o,
                                     exact=exact)
    # the workspace must be ready for the next call without re-initialisation
    ids_g2, lp_g2 = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws, tuning=tuning)
    _sync()
    assert torch.equal(ids_g, ids_g2) and torch.equal(lp_g, lp_g2)
    return frac, ids_g.cpu().numpy(), lp_g.cpu().numpy()


def test_tiny_config_draft_topk():
    c = CONFIGS["tiny"]
    _say("draft tiny config")
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(c.M, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    frac, _, _ = _run_draft(W, H, r, c.V_sub, c.k)
    _say("  rows identical to the oracle:", frac)


@pytest.mark.parametrize("M,d,V,V_sub,k", [
    (1, 256, 4096, 1024, 1), (10, 512, 6000, 3000, 10), (16, 256, 5000, 2500, 16),
    (5, 264, 3000, 777, 7), (10, 1024, 9000, 4099, 33), (3, 128, 2000, 1999, 64),
    (2, 64, 100, 10, 10), (10, 4096, 2000, 640, 10), (4, 8192, 3000, 1500, 8),
    # k = 11 .. 16: the bound of the folds and of the merge comes from 32 groups instead of 16
    (10, 512, 40000, 36000, 11), (10, 256, 70000, 66000, 12), (7, 512, 40000, 20000, 13),
    (12, 256, 40000, 33000, 14), (10, 512, 50000, 40960, 15), (16, 256, 70000, 65536, 16),
    (10, 128, 3000, 16, 16), (3, 256, 5000, 300, 15),
    # the two routing rules that depend on the rows of W per compute unit: long rows of H with a pass for
    # every compute unit (chunked kernel), 13 / 14 rows of H on a small subset (four-wavefront skinny build)
    (4, 5120, 33000, 32768, 10), (13, 4096, 9000, 8192, 10), (14, 2048, 14000, 12288, 7)])
def test_draft_topk_skinny(M, d, V, V_sub, k):
    _say("draft skinny", M, d, V, V_sub, k)
    W, H, r = _case(V, d, M, 5)
    frac, _, _ = _run_draft(W, H, r, V_sub, k)
    _say("  rows identical to the oracle (matrix cores):", frac)
    t = Tuning()
    t.path = 1
    frac, _, _ = _run_draft(W, H, r, V_sub, k, tuning=t)
    _say("  rows identical to the oracle (vector ALUs):", frac)


@pytest.mark.parametrize("M,d,V,V_sub,k", [
    (17, 256, 4096, 1024, 4), (60, 512, 6000, 3000, 10), (64, 256, 5000, 2500, 16),
    (100, 264, 3000, 777, 7), (256, 128, 3000, 1500, 10), (300, 64, 2000, 900, 5),
    (40, 128, 2000, 1999, 64), (10, 8192, 3000, 1500, 10), (33, 8192, 1200, 700, 16),
    (80, 256, 3000, 1500, 10), (96, 512, 2000, 1000, 12), (44, 4096, 1500, 1100, 10)])
def test_draft_topk_matrix_core(M, d, V, V_sub, k):
    _say("draft mfma", M, d, V, V_sub, k)
    W, H, r = _case(V, d, M, 6)
    frac, _, _ = _run_draft(W, H, r, V_sub, k)
    _say("  rows identical to the oracle:", frac)


# The block kernel takes 65 to 256 rows of H per launch when d is a multiple of 128 and k <= 16:
# its three builds (up to 128, 192 and 256 rows), vocabulary sizes that are no multiple of its
# 128-row pass, more rows than one launch holds, few workgroups (several passes per workgroup:
# the running lists compete), both merge routes, and the same calls through the chunked kernel.
_BLOCK_CASES = [
    (65, 128, 3000, 300, 10, {}), (128, 256, 5000, 2500, 16, {}), (129, 128, 3000, 1500, 1, {}),
    (192, 384, 4000, 1000, 10, {}), (200, 1024, 4000, 2048, 7, {}), (256, 256, 3000, 1500, 10, {}),
    (300, 128, 2000, 900, 5, {}), (600, 128, 1500, 640, 3, {}), (100, 256, 9000, 4099, 10, dict(grid=3)),
    (256, 128, 9000, 9000, 16, dict(grid=5)), (96, 512, 2000, 1000, 12, dict(two_launch=1)),
    (120, 256, 3000, 129, 10, dict(no_mailbox=1)), (70, 2048, 1000, 127, 4, {}), (256, 4096, 700, 700, 10, {})]


@pytest.mark.parametrize("M,d,V,V_sub,k,knobs", _BLOCK_CASES)
def test_draft_topk_block_kernel(M, d, V, V_sub, k, knobs):
    _say("draft block kernel", M, d, V, V_sub, k, knobs)
    W, H, r = _case(V, d, M, 60)
    t = Tuning(path=2, **knobs)
    frac, ids_b, lp_b = _run_draft(W, H, r, V_sub, k, tuning=t)
    _say("  rows identical to the oracle (block kernel):", frac)
    t = Tuning(path=2, chunked_only=1, **knobs)
    frac, ids_c, lp_c = _run_draft(W, H, r, V_sub, k, tuning=t)
    _say("  rows identical to the oracle (chunked kernel, slabs):", frac)


@pytest.mark.parametrize("M,k", [(80, 12), (256, 12), (130, 16)])
def test_draft_topk_block_kernel_exact_inputs_identical_with_ties(M, k):
    # integer-valued inputs, logits full of ties: the ids must match the oracle with no exemption
    # (the general fold and merge run where more than 32 candidates of a row tie)
    _say("draft block kernel, exact + ties", M, k)
    W_bits, H_bits, _, _ = make_exact_case(V=3000, d=128, M=M, seed=300 + M, w_levels=1, h_levels=1)
    r = np.random.default_rng(12).permutation(3000).astype(np.int32)
    frac, _, _ = _run_draft(W_bits, H_bits, r, 1500, k, exact=True)
    assert frac == 1.0


@pytest.mark.parametrize("M,d,V", [(65, 128, 129), (128, 4096, 300), (192, 256, 1000), (256, 512, 513), (600, 128, 260)])
def test_logits_block_kernel_exact_inputs_bit_exact(M, d, V):
    _say("logits block kernel, exact", M, d, V)
    W_bits, H_bits, W_int, H_int = make_exact_case(V=V, d=d, M=M, seed=M + V)
    exact = (H_int @ W_int.T).astype(np.float32)
    z_g = fr.fr_draft_logits(to_dev_bf16(H_bits), to_dev_bf16(W_bits))
    _sync()
    assert np.array_equal(z_g.cpu().numpy(), exact)


@pytest.mark.parametrize("M", [4, 10, 48])
def test_draft_topk_exact_inputs_identical_with_ties(M):
    # Integer-valued inputs: logits are exact on both sides and full of ties, so the
    # ids must match the oracle with no exemption (this pins the tie rule on the GPU).
    _say("draft exact + ties", M)
    W_bits, H_bits, _, _ = make_exact_case(V=3000, d=72, M=M, seed=100 + M, w_levels=1, h_levels=1)
    r = np.random.default_rng(11).permutation(3000).astype(np.int32)
    frac, _, _ = _run_draft(W_bits, H_bits, r, 1500, 12, exact=True)
    assert frac == 1.0


def test_duplicate_rows_tie_goes_to_lower_full_vocab_id():
    _say("draft duplicate rows")
    W, H, r = _case(4000, 256, 10, 8)
    # make the best token of every row of H a duplicate pair (higher id ranked first)
    W[3999] = W[17]
    H = f32_to_bf16_bits(np.tile(bf16_bits_to_f32(W[17]) * 8, (10, 1)))
    r = np.concatenate([[3999, 17], np.setdiff1d(np.arange(4000), [17, 3999])]).astype(np.int32)
    _, ids_g, lp_g = _run_draft(W, H, r, 2000, 4)
    assert np.all(ids_g[:, 0] == 17) and np.all(ids_g[:, 1] == 3999)
    assert np.array_equal(lp_g[:, 0], lp_g[:, 1])


@pytest.mark.parametrize("knobs", [dict(two_launch=1), dict(ksplit=2), dict(ksplit=8), dict(grid=3),
                                   dict(grid=1), dict(variant=2), dict(variant=3), dict(variant=4),
                                   dict(variant=5), dict(variant=6), dict(path=1), dict(path=1, ksplit=4),
                                   dict(path=1, two_launch=1), dict(path=2), dict(path=2, two_launch=1),
                                   dict(path=2, no_mailbox=1)])
def test_kernel_variants_agree(knobs):
    _say("variants", knobs)
    W, H, r = _case(6000, 512, 10, 9)
    base = _run_draft(W, H, r, 3000, 10)
    t = Tuning()
    for key, val in knobs.items():
        setattr(t, key, val)
    other = _run_draft(W, H, r, 3000, 10, tuning=t)
    # different summation orders may flip genuine near ties, nothing else
    same = base[1] == other[1]
    assert np.mean(same) > 0.9
    assert np.max(np.abs(base[2] - other[2])) < LOGIT_TOL


@pytest.mark.parametrize("M,k", [(10, 10), (64, 10)])
def test_full_topk_matches_oracle(M, k):
    _say("full topk", M, k)
    W, H, _ = _case(5003, 512, M, 10)
    ids_o, lp_o, z_o = oracle.full_topk(H, W, k, want_logits=True)
    ws = fr.new_workspace(M, 512, 5003, k)
    ids_g, lp_g = fr.fr_full_topk(to_dev_bf16(H), to_dev_bf16(W), k, ws)
    _sync()
    check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, None, ids_o, lp_o)


def test_v_sub_equal_v_draft_equals_full():
    _say("V_sub == V")
    W, H, _ = _case(2048, 256, 10, 12)
    ident = np.arange(2048, dtype=np.int32)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(ident), 2048)
    ws = fr.new_workspace(10, 256, 2048, 10)
    a = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, 10, ws)
    b = fr.fr_full_topk(to_dev_bf16(H), to_dev_bf16(W), 10, ws)
    _sync()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_nan_and_inf_inputs_do_not_hang():
    _say("nan / inf inputs")
    W, H, r = _case(2000, 128, 4, 13)
    W[5, 3] = 0x7FC0    # NaN
    W[9, 1] = 0x7F80    # +inf
    H[1, 0] = 0xFF80    # -inf
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), 1000)
    ws = fr.new_workspace(4, 128, 1000, 5)
    ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, 5, ws)
    _sync()
    assert ids_g.shape == (4, 5)


def test_workspace_reuse_with_changing_inputs_sees_no_stale_partials():
    # The single-launch merge reads partials written by workgroups on other compute dies.
    # Reusing one workspace for different inputs, back to back, would expose a merge that
    # reads the previous call's partials.
    _say("workspace reuse, changing inputs")
    W, _, r = _case(8000, 512, 10, 14)
    V_sub, k = 4096, 10
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(10, 512, V_sub, k)
    g = np.random.default_rng(15)
    Hs = [f32_to_bf16_bits(g.standard_normal((10, 512)).astype(np.float32)) for _ in range(8)]
    Hd = [to_dev_bf16(h) for h in Hs]
    outs = [fr.fr_draft_topk(h, W_g, idx_g, k, ws) for h in Hd]   # enqueued back to back
    _sync()
    for h, (ids_g, lp_g) in zip(Hs, outs):
        ids_o, lp_o, z_o = oracle.draft_topk(h, W_o, idx_o, k, want_logits=True)
        check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)


def test_one_workspace_across_changing_shapes_leaves_the_mailbox_empty():
    # The single-launch merge (skinny kernel, chunked kernel up to 128 rows of H, block kernel up to 256)
    # passes results through self-validating records that must all be empty again when a
    # call ends, whatever M, k, the kernel and the number of workgroups were; a record left
    # behind would be taken for a result by a later call.
    _say("workspace reuse, changing shapes")
    W, _, r = _case(9000, 256, 16, 21)
    ws = fr.new_workspace(256, 256, 9000, 16)
    W_d, r_d = to_dev_bf16(W), to_dev_i32(r)
    g = np.random.default_rng(22)
    shapes = [(10, 10, 4096, {}), (3, 16, 9000, {}), (16, 1, 100, {}), (10, 10, 4096, dict(grid=5)),
              (1, 7, 2048, dict(ksplit=2)), (12, 12, 6000, {}), (10, 10, 4096, dict(path=1)), (16, 16, 9000, {}),
              (40, 10, 4096, {}), (10, 10, 4096, dict(path=2)), (64, 16, 9000, {}), (17, 3, 300, {}),
              (40, 10, 4096, dict(no_mailbox=1)), (33, 1, 9000, dict(grid=7)), (100, 10, 9000, {}),
              (128, 16, 4096, {}), (90, 5, 9000, dict(grid=9)), (10, 10, 4096, {}), (256, 10, 9000, {}),
              (200, 16, 4096, dict(grid=6)), (130, 3, 700, {}), (10, 10, 4096, {})]
    for rep in range(2):
        for M, k, V_sub, knobs in shapes:
            H = f32_to_bf16_bits(g.standard_normal((M, 256)).astype(np.float32))
            W_o, idx_o = oracle.build_subset(W, r, V_sub)
            ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
            W_g, idx_g = fr.fr_build_subset(W_d, r_d, V_sub)
            t = None
            if knobs:
                t = Tuning()
                for key, val in knobs.items():
                    setattr(t, key, val)
            ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws, tuning=t)
            _sync()
            check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
            mail = ws[512:512 + (256 * 16 + 256) * 512 * 8].cpu().numpy()
            assert (mail == 0xFF).all(), (M, k, V_sub, knobs)
            head = ws[:512].cpu().numpy().view(np.uint32)
            assert head[1] == 0      # no wait ever timed out
    assert fr.fr_workspace_check(ws) is False


@pytest.mark.parametrize("M,k,skew,exact", [(10, 10, 4, False), (10, 10, 8, False), (10, 10, 16, False),
                                            (10, 10, 0, False), (1, 1, 4, False), (12, 16, 12, False),
                                            (7, 20, 4, False), (10, 10, 4, True), (3, 33, 16, True)])
def test_skewed_rows_between_neighbouring_workgroups(M, k, skew, exact):
    # 32768 rows = one pass of 128 rows for each of the 256 workgroups: the only shape at which
    # the skinny kernel moves rows from odd to even workgroups (a ninth wavefront streams the
    # surplus).  `exact` inputs give heavily tied logits: the general fold and merge run.
    _say("skewed build", M, k, skew, exact)
    V, V_sub, d = 40000, 32768, 128
    if exact:
        W, H = make_exact_case(V, d, M, 31)[:2]
    else:
        W = make_weights(V, d, 30)
        H = make_hidden(M, d, 30)
    r = np.random.default_rng([20250214, 94]).permutation(V).astype(np.int32)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V, k)
    t = Tuning()
    t.skew = skew
    ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws, tuning=t)
    _sync()
    check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
    assert fr.fr_workspace_check(ws) is False


@pytest.mark.parametrize("n_blocks,rows,k", [(4, 1, 10), (5, 3, 10), (2, 8, 16), (1, 10, 10), (3, 20, 10)])
def test_hidden_states_in_several_blocks(n_blocks, rows, k):
    # fr_draft_topk_multi: the rows of H sit in separately allocated blocks (several draft heads
    # against one W_sub); the result must be what the stacked problem gives, bit for bit for the
    # single-launch path (the kernel sees the same rows in the same order).
    _say("several blocks of hidden states", n_blocks, rows, k)
    V, V_sub, d = 6000, 3000, 512
    W, _, r = _case(V, d, 1, 41)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    blocks = [make_hidden(rows, d, 50 + b) for b in range(n_blocks)]
    pads = [torch.empty(1000 * (b + 1), device="cuda") for b in range(n_blocks)]   # keep the blocks apart
    dev = [to_dev_bf16(h) for h in blocks]
    H_all = np.concatenate(blocks, axis=0)
    M = n_blocks * rows
    ws = fr.new_workspace(M, d, V, k)
    ids_m, lp_m = fr.fr_draft_topk_multi(dev, W_g, idx_g, k, ws)
    ids_s, lp_s = fr.fr_draft_topk(to_dev_bf16(H_all), W_g, idx_g, k, ws)
    _sync()
    ids_o, lp_o, z_o = oracle.draft_topk(H_all, W_o, idx_o, k, want_logits=True)
    check_topk_against_oracle(ids_m.cpu().numpy(), lp_m.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
    if M <= 16:
        assert np.array_equal(ids_m.cpu().numpy(), ids_s.cpu().numpy())
        assert np.array_equal(lp_m.cpu().numpy().view(np.uint32), lp_s.cpu().numpy().view(np.uint32))
    del pads


@pytest.mark.parametrize("knobs,M,k", [(dict(), 10, 10), (dict(path=2), 40, 10), (dict(), 10, 20),
                                       (dict(path=2, no_mailbox=1), 24, 10)])
def test_a_wait_that_runs_out_reports_no_result_and_the_workspace_recovers(knobs, M, k):
    # The waits inside the single-launch merge are bounded.  Here the bound is forced down to one
    # poll from the host, so that a merger gives up (every kernel still ends normally): the
    # subset is one 128-row pass longer than one pass per compute unit, so the first workgroup
    # streams twice as long as the mergers, which sit at the end of the grid.  Per row either
    # outcome is accepted: the result of an ordinary call, or "no result" (id INT32_MAX,
    # logp -inf) together with the sticky word.  After fr_workspace_init the workspace works again.
    _say("forced time-out", knobs, M, k)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    d, V_sub = 4096, 128 * cus + 128
    V = V_sub + 100
    W, H, r = _case(V, d, M, 31)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    H_d = to_dev_bf16(H)
    ws = fr.new_workspace(M, d, V, k)
    ids_ref, lp_ref = fr.fr_draft_topk(H_d, W_g, idx_g, k, ws)
    _sync()
    ids_ref, lp_ref = ids_ref.cpu().numpy(), lp_ref.cpu().numpy()
    t = Tuning(spin_limit=1, **knobs)
    gave_up = 0
    for rep in range(3):
        ids_g, lp_g = fr.fr_draft_topk(H_d, W_g, idx_g, k, ws, tuning=t)
        _sync()
        ids_g, lp_g = ids_g.cpu().numpy(), lp_g.cpu().numpy()
        timed_out = fr.fr_workspace_check(ws)
        none = 0
        for m in range(M):
            if np.all(ids_g[m] == np.iinfo(np.int32).max):
                assert np.all(np.isneginf(lp_g[m])), (m, lp_g[m])
                none += 1
            else:
                assert np.array_equal(ids_g[m], ids_ref[m]) and np.array_equal(lp_g[m], lp_ref[m]), m
        assert (none > 0) == timed_out or (timed_out and none == 0)   # no sentinel row without the word
        assert none == 0 or timed_out
        gave_up += none
        fr.fr_workspace_init(ws)
        _sync()
        assert fr.fr_workspace_check(ws) is False
    _say("  rows that reported no result over 3 calls:", gave_up)
    assert gave_up > 0
    ids_g, lp_g = fr.fr_draft_topk(H_d, W_g, idx_g, k, ws)
    _sync()
    assert np.array_equal(ids_g.cpu().numpy(), ids_ref) and np.array_equal(lp_g.cpu().numpy(), lp_ref)
    assert fr.fr_workspace_check(ws) is False
