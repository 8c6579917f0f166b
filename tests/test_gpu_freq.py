"""GPU parity of the corpus-statistics kernels (token counting, frequency ranking) against
the CPU oracle: integer work, compared bit for bit."""

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14856_amd as fr

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _zipf_stream(rng, V, n, s=1.1):
    p = 1.0 / np.arange(1, V + 1) ** s
    p /= p.sum()
    perm = rng.permutation(V)
    return perm[rng.choice(V, size=n, p=p)].astype(np.int32)


@pytest.mark.parametrize("V,n", [(1000, 0), (1000, 3), (1000, 1027), (50000, 200001), (128256, 1 << 20),
                                 (152064, 777777), (32768, 65536), (32769, 65537)])
def test_count_tokens_matches_oracle(V, n):
    _say("count tokens", V, n)
    rng = np.random.default_rng([20250214, 97, V, n])
    tokens = _zipf_stream(rng, V, n) if n else np.zeros(0, np.int32)
    want, _ = oracle.count_tokens(tokens, V)
    t_d = torch.from_numpy(tokens).cuda() if n else torch.zeros(4, dtype=torch.int32, device="cuda")[:0]
    got = fr.fr_count_tokens(t_d, V)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)


def test_count_tokens_accumulates_and_flags_bad_ids():
    V = 70000
    rng = np.random.default_rng([20250214, 98])
    a, b = _zipf_stream(rng, V, 300001), _zipf_stream(rng, V, 99999)
    b[::1000] = V + 5
    b[1::1000] = -1
    want, _ = oracle.count_tokens(a, V)
    want, bad = oracle.count_tokens(b, V, want)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    counts = fr.fr_count_tokens(torch.from_numpy(a).cuda(), V, dev_error_flag=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    fr.fr_count_tokens(torch.from_numpy(b).cuda(), V, counts=counts, dev_error_flag=flag)
    torch.cuda.synchronize()
    assert bad > 0 and int(flag.item()) == 1
    assert np.array_equal(counts.cpu().numpy(), want)


# ("edges": counts on both sides of every boundary between the count-magnitude buckets that the
# ranking deals the ids into; "equal": one bucket holds everything)
@pytest.mark.parametrize("V,kind", [(1, "zero"), (257, "ties"), (5000, "ties"), (128256, "zipf"), (152064, "ties"),
                                    (4099, "big"), (20011, "edges"), (70001, "equal"), (300000, "zipf")])
def test_rank_tokens_matches_oracle(V, kind):
    _say("rank tokens", V, kind)
    rng = np.random.default_rng([20250214, 99, V])
    if kind == "zero":
        counts = np.zeros(V, np.int64)
    elif kind == "ties":
        counts = rng.integers(0, 25, size=V).astype(np.int64)
    elif kind == "edges":
        e = rng.integers(0, 62, size=V)
        mant = rng.integers(0, 33, size=V)
        base = (np.int64(1) << e) + ((mant.astype(np.int64) << e) >> 5)
        counts = np.maximum(base + rng.integers(-1, 2, size=V), 0).astype(np.int64)
    elif kind == "equal":
        counts = np.full(V, 5, np.int64)
    elif kind == "big":
        counts = rng.integers(0, 1 << 62, size=V).astype(np.int64)
        counts[::7] = counts[3]
    else:
        counts, _ = oracle.count_tokens(_zipf_stream(rng, V, 1 << 20), V)
    want = oracle.rank_tokens(counts)
    got = fr.fr_rank_tokens(torch.from_numpy(counts).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)


def test_counts_to_subset_end_to_end():
    # stream -> counts -> ranking -> gather: the ranking produced on the GPU drives Eq. 3
    from parity_utils import bits_of, to_dev_bf16
    from synth import make_weights
    V, d, V_sub = 8192, 256, 2048
    rng = np.random.default_rng([20250214, 100])
    tokens = _zipf_stream(rng, V, 500000)
    ranked_g = fr.fr_rank_tokens(fr.fr_count_tokens(torch.from_numpy(tokens).cuda(), V))
    W = make_weights(V, d, 8)
    W_g, idx_g = fr.fr_build_subset(to_dev_bf16(W), ranked_g, V_sub)
    torch.cuda.synchronize()
    ranked_o = oracle.rank_tokens(oracle.count_tokens(tokens, V)[0])
    W_o, idx_o = oracle.build_subset(W, ranked_o, V_sub)
    assert np.array_equal(idx_g.cpu().numpy(), idx_o) and np.array_equal(bits_of(W_g), W_o)
