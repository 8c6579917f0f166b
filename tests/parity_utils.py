"""Helpers shared by the GPU parity tests: tensor marshalling and the comparison rules.

Comparison bar (stated with the build's target): subset gather and id remap bit-exact;
logits within max-abs 1e-2 of the oracle's fp32 logits; top-k ids identical except
where the oracle's logits of the two tokens involved differ by less than 1e-2.
"""

import numpy as np
import torch

LOGIT_TOL = 1e-2
# What the arithmetic gives (fp32 accumulation of d <= 4096 exact products, fast exp/log in the
# normaliser): the full-size tests assert this tighter band beside the 1e-2 bar.
TIGHT_TOL = 1e-4


class ParityReport(float):
    """The fraction of rows whose ids equal the oracle's, carrying the achieved errors."""
    logp_err = 0.0     # max |logp_gpu - (z*_oracle[id] - logZ_oracle)| over all returned entries



def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> CUDA bfloat16 tensor with the same bits."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_dev_i32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def check_topk_against_oracle(ids_g, logp_g, z_star, idx_map, ids_o, logp_o, tol=LOGIT_TOL,
                              exact=False, logp_tight=None):
    """ids_g/logp_g: GPU output [M,k]; z_star: oracle fp32 logits [M,rows];
    idx_map: position -> id (None = identity); ids_o/logp_o: oracle output.
    Returns the fraction of rows whose ids match the oracle exactly (a ParityReport: its
    logp_err is the largest log-probability error seen); with logp_tight, that error must
    also stay below logp_tight."""
    M, k = ids_g.shape
    rows = z_star.shape[1]
    ids_of_pos = np.arange(rows, dtype=np.int64) if idx_map is None else idx_map.astype(np.int64)
    pos_of_id = {}
    exact_rows = 0
    lz = None
    logp_err = 0.0
    for m in range(M):
        if exact:
            assert np.array_equal(ids_g[m], ids_o[m]), (m, ids_g[m], ids_o[m])
        if not pos_of_id:
            pos_of_id = {int(t): i for i, t in enumerate(ids_of_pos)}
        g = [int(t) for t in ids_g[m]]
        # (1) distinct members of the subset
        assert len(set(g)) == k, (m, g)
        assert all(t in pos_of_id for t in g), (m, g)
        zg = np.array([z_star[m, pos_of_id[t]] for t in g], dtype=np.float64)
        zo = np.array([z_star[m, pos_of_id[int(t)]] for t in ids_o[m]], dtype=np.float64)
        # (2) position-wise the same token, or a near tie in the oracle's own logits
        for j in range(k):
            assert g[j] == int(ids_o[m, j]) or abs(zg[j] - zo[j]) < tol, (m, j, g[j], ids_o[m, j], zg[j], zo[j])
        # (3) nothing below the oracle's k-th logit by more than the tolerance
        assert np.all(zg >= zo[-1] - tol), (m, zg, zo[-1])
        # (4) log-probabilities of the returned tokens
        lz = float(zo[0]) - float(logp_o[m, 0])   # oracle's log Z of this row
        err = float(np.max(np.abs(logp_g[m].astype(np.float64) - (zg - lz))))
        assert err <= tol, (m, logp_g[m], zg - lz)
        if logp_tight is not None:
            assert err < logp_tight, (m, err, logp_g[m], zg - lz)
        logp_err = max(logp_err, err)
        # (5) the GPU's own order
        assert np.all(np.diff(logp_g[m]) <= 0), (m, logp_g[m])
        exact_rows += int(np.array_equal(ids_g[m], ids_o[m]))
    report = ParityReport(exact_rows / M)
    report.logp_err = logp_err
    return report
