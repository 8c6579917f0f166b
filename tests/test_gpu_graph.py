"""A whole draft phase (six draft LM-head calls with their beam-search expansion, then the
draft-tree selection; Section 2 and Section 4.1: depth 6, 60 draft tokens) captured once in a
HIP graph and replayed.  The library keeps its state (arrival turn, result mailbox) in the
caller's workspace and launches nothing but kernels, so a replay must give, bit for bit, what
the same calls give when issued one by one; each replay is checked, with eager calls on the
same workspace in between."""

import numpy as np
import pytest
import torch

import paper_2502_14856_amd as fr
from parity_utils import to_dev_bf16, to_dev_i32
from synth import make_hidden, make_weights, zipf_ranking

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("fused", [False, True])
def test_draft_phase_replayed_from_a_graph_equals_the_eager_calls(fused):
    _say("graph replay of a draft phase, fused steps:", fused)
    d, V, V_sub, k, width, depth, K = 512, 8192, 4096, 10, 10, 6, 60
    W = make_weights(V, d, 0)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 0)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(width, d, V, k)
    cap = k + (depth - 1) * width * k
    i32 = dict(dtype=torch.int32, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")

    # every buffer the phase touches exists before the capture
    rows = [1] + [width] * (depth - 1)
    H = [torch.zeros((m, d), dtype=torch.bfloat16, device="cuda") for m in rows]
    ids = [torch.empty((m, k), **i32) for m in rows]
    lp = [torch.empty((m, k), **f32) for m in rows]
    hist = [torch.zeros(cap, **f32), torch.zeros(cap, **i32), torch.zeros(cap, **i32)]
    ns = [torch.zeros(1, **f32)] + [torch.empty(width, **f32) for _ in range(depth)]
    nt = [None] + [torch.empty(width, **i32) for _ in range(depth)]
    nh = [torch.full((1,), -1, **i32)] + [torch.empty(width, **i32) for _ in range(depth)]
    sel = [torch.empty(K, **i32) for _ in range(4)] + [torch.empty((K, K), dtype=torch.uint8, device="cuda")]

    def phase():
        off = 0
        for s, m in enumerate(rows):
            w = min(width, m * k)
            if fused:
                fr.fr_draft_step(H[s], W_g, idx_g, k, ns[s][:m], nh[s][:m], w, *hist, off, ws, token_ids=ids[s],
                                 logp=lp[s], next_score=ns[s + 1][:w], next_token=nt[s + 1][:w],
                                 next_hist=nh[s + 1][:w])
            else:
                fr.fr_draft_topk(H[s], W_g, idx_g, k, ws, token_ids=ids[s], logp=lp[s])
                fr.fr_beam_expand(lp[s], ids[s], ns[s][:m], nh[s][:m], w, *hist, off, next_score=ns[s + 1][:w],
                                  next_token=nt[s + 1][:w], next_hist=nh[s + 1][:w])
            off += m * k
        fr.fr_tree_select(*hist, off, K, out=sel)

    def load_inputs(case):
        for s, m in enumerate(rows):
            H[s].copy_(to_dev_bf16(make_hidden(m, d, 300 + 10 * case + s)))

    def snapshot():
        torch.cuda.synchronize()
        return [t.cpu().numpy().copy() for t in hist + sel + ids + lp]

    # eager results for two sets of hidden states (also the warm-up that a capture needs)
    want = []
    for case in range(2):
        load_inputs(case)
        phase()
        want.append(snapshot())
    assert not all(np.array_equal(a, b) for a, b in zip(*want))   # the two cases do differ

    fr.fr_init()                       # the per-device set-up never happens inside a capture
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):      # the binding launches on torch's current stream: the capturing one
        phase()
    torch.cuda.synchronize()

    H_other = to_dev_bf16(make_hidden(width, d, 999))
    for replay, case in enumerate([0, 1, 1, 0, 1]):
        load_inputs(case)
        for t in hist + sel + ids + lp:
            t.zero_()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want[case]):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), (replay, case)
        # the program's own eager work on the same workspace between two replays
        fr.fr_draft_topk(H_other, W_g, idx_g, k, ws)
        torch.cuda.synchronize()
    assert fr.fr_workspace_check(ws) is False


@pytest.mark.parametrize("M", [40, 100, 200])
def test_chunked_kernel_replayed_from_a_graph_equals_the_eager_call(M):
    # the chunked kernel's single-launch merge (40 and 100 rows of H: result mailbox) and its
    # slabs (200 rows: two launches), captured and replayed with other calls in between
    _say("graph replay of the chunked kernel, rows of H:", M)
    d, V, V_sub, k = 256, 6000, 3000, 10
    W = make_weights(V, d, 1)
    r, _ = zipf_ranking(V, 1.1, 10 ** 6, 1)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), to_dev_i32(r), V_sub)
    ws = fr.new_workspace(M, d, V, k)
    H = torch.zeros((M, d), dtype=torch.bfloat16, device="cuda")
    ids = torch.empty((M, k), dtype=torch.int32, device="cuda")
    lp = torch.empty((M, k), dtype=torch.float32, device="cuda")
    want = []
    for case in range(2):
        H.copy_(to_dev_bf16(make_hidden(M, d, 500 + case)))
        fr.fr_draft_topk(H, W_g, idx_g, k, ws, token_ids=ids, logp=lp)
        torch.cuda.synchronize()
        want.append((ids.cpu().numpy().copy(), lp.cpu().numpy().copy()))
    assert not np.array_equal(want[0][0], want[1][0])
    fr.fr_init()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fr.fr_draft_topk(H, W_g, idx_g, k, ws, token_ids=ids, logp=lp)
    torch.cuda.synchronize()
    H_other = to_dev_bf16(make_hidden(10, d, 998))
    for replay, case in enumerate([1, 0, 0, 1]):
        H.copy_(to_dev_bf16(make_hidden(M, d, 500 + case)))
        ids.zero_()
        lp.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), want[case][0]), (replay, case)
        assert np.array_equal(lp.cpu().numpy().view(np.uint32), want[case][1].view(np.uint32)), (replay, case)
        fr.fr_draft_topk(H_other, W_g, idx_g, k, ws)
        torch.cuda.synchronize()
    assert fr.fr_workspace_check(ws) is False
