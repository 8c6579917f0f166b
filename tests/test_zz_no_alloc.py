"""fr_draft_topk_static, the entry point for callers that cannot allocate (its workspace is a
static array in device memory), against fr_draft_topk on a caller's workspace: the same
kernels on another buffer, so the outputs must agree bit for bit; two calls in a row on the
shared scratch, the second one smaller."""

import numpy as np
import pytest
import torch

import paper_2502_14856_amd as fr
from parity_utils import to_dev_bf16, to_dev_i32
from synth import make_hidden, make_weights, zipf_ranking

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _both(H_d, W_g, idx_g, k, ws):
    M = H_d.shape[0]
    ids_r, lp_r = fr.fr_draft_topk(H_d, W_g, idx_g, k, ws)
    ids_s = torch.full((M, k), -5, dtype=torch.int32, device="cuda")
    lp_s = torch.full((M, k), 5.0, dtype=torch.float32, device="cuda")
    fr.fr_draft_topk_static(H_d, W_g, idx_g, k, ids_s, lp_s)
    torch.cuda.synchronize()
    assert np.array_equal(ids_s.cpu().numpy(), ids_r.cpu().numpy())
    assert np.array_equal(lp_s.cpu().numpy().view(np.uint32), lp_r.cpu().numpy().view(np.uint32))


@pytest.mark.parametrize("d,V,shapes", [
    (1024, 24000, [(10, 10, 20000), (4, 5, 3000), (16, 16, 24000), (1, 1, 17)]),   # skinny kernel
    (4096, 9000, [(16, 10, 8200), (13, 3, 700), (10, 10, 8200)]),                  # chunked kernel, then skinny
])
def test_static_scratch_calls_equal_workspace_calls(d, V, shapes):
    _say("no-alloc entry point", d, V, shapes)
    W = make_weights(V, d, 5)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 5)
    W_d, r_d = to_dev_bf16(W), to_dev_i32(r)
    for M, k, V_sub in shapes:                       # consecutive calls share the device's scratch
        _say("  M, k, V_sub =", M, k, V_sub)
        W_g, idx_g = fr.fr_build_subset(W_d, r_d, V_sub)
        ws = fr.new_workspace(M, d, V, k)
        _both(to_dev_bf16(make_hidden(M, d, 400 + M)), W_g, idx_g, k, ws)
        assert fr.fr_workspace_check(ws) is False


def test_fr_init_prepares_the_scratch_again():
    d, V, V_sub, M, k = 512, 4096, 2048, 8, 8
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(make_weights(V, d, 6)), to_dev_i32(zipf_ranking(V, 1.1, 10 ** 6, 6)[0]),
                                    V_sub)
    H_d = to_dev_bf16(make_hidden(M, d, 500))
    ws = fr.new_workspace(M, d, V, k)
    _both(H_d, W_g, idx_g, k, ws)
    fr.fr_init()                                     # nothing in flight: the scratch is prepared afresh
    _both(H_d, W_g, idx_g, k, ws)


def test_static_scratch_refuses_what_it_cannot_hold():
    L = fr.lib()
    SCRATCH = -6
    # fake pointers: nothing may be launched
    assert L.fr_draft_topk_static(0x1000, 17, 4096, 0x2000, 0, 32768, 10, 0x3000, 0x4000, None) == SCRATCH
    assert L.fr_draft_topk_static(0x1000, 10, 4096, 0x2000, 0, 32768, 17, 0x3000, 0x4000, None) == SCRATCH
    assert L.fr_draft_topk_static(0, 10, 4096, 0x2000, 0, 32768, 10, 0x3000, 0x4000, None) == -1
    assert "static scratch" in fr.fr_strerror(SCRATCH)
