"""GPU parity of the tiled-layout path: fr_build_subset_tiled is the gather of Eq. 3 stored in
another order (compared bit for bit after undoing the documented permutation), and
fr_draft_topk_tiled must give what fr_draft_topk gives (compared with the oracle to the same
bar as the row-major path)."""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr
from paper_2502_14856_amd.binding import Tuning
from parity_utils import bits_of, check_topk_against_oracle, to_dev_bf16, to_dev_i32
from synth import CONFIGS, make_hidden, make_weights, zipf_ranking

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def untile(flat_bits, V_sub, d):
    """Row-major [V_sub, d] view of a tiled W_sub.  Layout only (the formula of frspec.h):
    element (r, c) lives at (r/16)*16*d + (c/32)*512 + ((c%32)/8)*128 + (r%16)*8 + c%8."""
    tiles = (V_sub + 15) // 16
    a = flat_bits.reshape(tiles, d // 32, 4, 16, 8)        # tile, kb, g, i, e
    a = a.transpose(0, 3, 1, 2, 4).reshape(tiles * 16, d)  # (tile, i) rows; (kb, g, e) columns
    return a[:V_sub], a[V_sub:]


@pytest.mark.parametrize("V,d,V_sub", [(3000, 256, 2048), (3000, 256, 1000), (5003, 384, 5003), (600, 128, 17)])
def test_tiled_gather_is_the_gather_in_another_order(V, d, V_sub):
    _say("tiled gather", V, d, V_sub)
    W = make_weights(V, d, 3)
    r = np.random.default_rng([20250214, 93, V_sub]).permutation(V).astype(np.int32)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    W_t, idx_g = fr.fr_build_subset_tiled(to_dev_bf16(W), to_dev_i32(r), V_sub)
    torch.cuda.synchronize()
    assert W_t.numel() * 2 == fr.fr_tiled_bytes(V_sub, d)
    rows, pad = untile(bits_of(W_t), V_sub, d)
    assert np.array_equal(rows, W_o)
    assert not pad.any()
    assert np.array_equal(idx_g.cpu().numpy(), idx_o)


def test_tiled_gather_flags_bad_ids():
    V, d, V_sub = 500, 128, 40
    W = make_weights(V, d, 4)
    r = np.arange(V_sub, dtype=np.int32)
    r[5], r[33] = -3, V
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    W_t, idx_g = fr.fr_build_subset_tiled(to_dev_bf16(W), to_dev_i32(r), V_sub, dev_error_flag=flag)
    torch.cuda.synchronize()
    rows, _ = untile(bits_of(W_t), V_sub, d)
    assert int(flag.item()) == 1
    idx = idx_g.cpu().numpy()
    assert idx[5] == -1 and idx[33] == -1 and not rows[5].any() and not rows[33].any()
    good = np.setdiff1d(np.arange(V_sub), [5, 33])
    assert np.array_equal(rows[good], W[r[good]])


@pytest.mark.parametrize("V,d,V_sub,M,k,knobs", [
    (6000, 512, 3000, 10, 10, {}),
    (6000, 512, 2999, 10, 10, {}),                 # ragged last tile
    (6000, 512, 3000, 1, 1, {}),
    (6000, 512, 3000, 16, 16, {}),
    (6000, 512, 3000, 10, 10, dict(variant=8)),    # 6 stages
    (6000, 512, 3000, 10, 10, dict(variant=9)),    # 8 stages
    (6000, 512, 3000, 10, 10, dict(ksplit=4)),
    (6000, 512, 3000, 10, 10, dict(ksplit=1, grid=3)),   # several passes per workgroup
    (6000, 512, 3000, 10, 10, dict(two_launch=1)),
    (6000, 512, 3000, 7, 33, {}),                  # general fold and merge (k > 16)
    (4000, 128, 100, 4, 4, {}),
])
def test_tiled_draft_matches_oracle(V, d, V_sub, M, k, knobs):
    _say("tiled draft", V, d, V_sub, M, k, knobs)
    W = make_weights(V, d, 5)
    H = make_hidden(M, d, 5)
    r, _ = zipf_ranking(V, 1.1, 10 ** 5, 5)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
    W_t, idx_g = fr.fr_build_subset_tiled(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V, k)
    t = None
    if knobs:
        t = Tuning()
        for key, val in knobs.items():
            setattr(t, key, val)
    ids_g, lp_g = fr.fr_draft_topk_tiled(to_dev_bf16(H), W_t, idx_g, V_sub, k, ws, tuning=t)
    torch.cuda.synchronize()
    check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)


def test_tiled_draft_full_size_llama3_8b():
    c = CONFIGS["llama3_8b"]
    _say("tiled draft, full size")
    W = make_weights(c.V, c.d, c.index)
    H = make_hidden(c.M, c.d, c.index)
    r, _ = zipf_ranking(c.V, c.zipf_s, c.n_tokens, c.index)
    W_o, idx_o = oracle.build_subset(W, r, c.V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, c.k, want_logits=True)
    W_d, r_d = to_dev_bf16(W), to_dev_i32(r)
    W_t, idx_g = fr.fr_build_subset_tiled(W_d, r_d, c.V_sub)
    torch.cuda.synchronize()
    rows, _ = untile(bits_of(W_t), c.V_sub, c.d)
    assert np.array_equal(rows, W_o)
    ws = fr.new_workspace(c.M, c.d, c.V, c.k)
    ids_g, lp_g = fr.fr_draft_topk_tiled(to_dev_bf16(H), W_t, idx_g, c.V_sub, c.k, ws)
    torch.cuda.synchronize()
    frac = check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
    _say("  rows identical to the oracle:", frac)


def test_tiled_entry_refuses_what_it_cannot_do():
    UNSUPPORTED = -5
    L = fr.lib()
    assert fr.fr_tiled_bytes(100, 4096) == 112 * 4096 * 2
    assert fr.fr_tiled_bytes(100, 200) == 0
    # fake pointers: nothing may be launched
    assert L.fr_draft_topk_tiled(0x1000, 17, 4096, 0x2000, 0, 32768, 10, 0x3000, 0x4000, 0x5000, 1 << 26, None,
                                 None) == UNSUPPORTED
    assert L.fr_draft_topk_tiled(0x1000, 10, 4096 + 64, 0x2000, 0, 32768, 10, 0x3000, 0x4000, 0x5000, 1 << 26,
                                 None, None) == UNSUPPORTED
