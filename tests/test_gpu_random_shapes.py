"""GPU parity on seeded random shapes: every routing boundary of the library (skinny kernel up to 16
rows of H, chunked kernel up to 64, block kernel up to 256 per launch where d is a multiple of 128 and
k <= 16, slabs beyond; threshold selection up to k = 16, general selection beyond; subsets smaller
than a pass, than the device, and several passes per workgroup) is crossed by some case; each case
is compared with the oracle to the bar of the other parity tests."""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr
from parity_utils import LOGIT_TOL, check_topk_against_oracle, to_dev_bf16, to_dev_i32
from synth import f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def _shapes(n, seed):
    g = np.random.default_rng([20250214, seed])
    out = []
    for _ in range(n):
        M = int(g.choice([1, 2, 7, 10, 12, 13, 16, 17, 31, 48, 64, 65, 66, 100, 127, 128, 129, 191, 193, 256, 257, 300]))
        d = int(g.choice([8, 64, 72, 128, 256, 264, 384, 520, 1024]))
        V = int(g.integers(40, 6000))
        V_sub = int(g.integers(max(1, V // 8), V + 1))
        k = int(g.choice([1, 3, 10, 16, 17, 40]))
        k = min(k, V_sub)
        out.append((M, d, V, V_sub, k))
    return out


@pytest.mark.parametrize("M,d,V,V_sub,k", _shapes(36, 1))
def test_random_shape_matches_oracle(M, d, V, V_sub, k):
    print("random shape", M, d, V, V_sub, k, flush=True)
    g = np.random.default_rng([M, d, V, V_sub, k])
    W = f32_to_bf16_bits((g.standard_normal((V, d)) * 0.05).astype(np.float32))
    H = f32_to_bf16_bits(g.standard_normal((M, d)).astype(np.float32))
    r = g.permutation(V).astype(np.int32)
    W_o, idx_o = oracle.build_subset(W, r, V_sub)
    ids_o, lp_o, z_o = oracle.draft_topk(H, W_o, idx_o, k, want_logits=True)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V_sub, k)
    ids_g, lp_g = fr.fr_draft_topk(to_dev_bf16(H), W_g, idx_g, k, ws)
    z_g = fr.fr_draft_logits(to_dev_bf16(H), W_g)
    torch.cuda.synchronize()
    assert np.array_equal(idx_g.cpu().numpy(), idx_o)
    assert float(np.max(np.abs(z_g.cpu().numpy() - z_o))) <= LOGIT_TOL
    check_topk_against_oracle(ids_g.cpu().numpy(), lp_g.cpu().numpy(), z_o, idx_o, ids_o, lp_o)
    assert fr.fr_workspace_check(ws) is False
