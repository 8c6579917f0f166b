"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, sizes workspaces, and rejects bad arguments before launching anything."""

import ctypes
import os
import re

import pytest

import paper_2502_14856_amd as fr
from paper_2502_14856_amd.binding import Tuning

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include")))
           if n.endswith(".h")]

INVALID, ALIGN, WORKSPACE, UNSUPPORTED = -1, -2, -3, -5


def _declared_symbols():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(fr_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_product_header_carries_no_measurement_surface():
    # knobs, traces and calibration kernels are declared in frspec_dev.h only
    text = open(os.path.join(ROOT, "include", "frspec.h")).read()
    for word in ("fr_tuning", "fr_calib_", "_tuned", "trace"):
        assert word not in text, word


def test_library_exports_every_declared_symbol():
    L = fr.lib()
    names = _declared_symbols()
    assert {"fr_build_subset", "fr_draft_topk", "fr_full_topk", "fr_workspace_bytes",
            "fr_workspace_init", "fr_strerror", "fr_init", "fr_draft_topk_tuned", "fr_calib_read"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_strerror_and_version():
    assert fr.fr_version() >= 101
    assert fr.fr_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert fr.fr_strerror(code)


def test_workspace_bytes_is_pure_host_arithmetic():
    a = fr.fr_workspace_bytes(10, 4096, 32768, 10)
    assert a > 0 and a % 256 == 0
    assert fr.fr_workspace_bytes(10, 4096, 128256, 10) == a     # independent of the rows read
    assert fr.fr_workspace_bytes(16, 4096, 32768, 10) > a
    assert fr.fr_workspace_bytes(10, 4096, 32768, 64) > a
    assert fr.fr_workspace_bytes(1000, 4096, 32768, 10) == fr.fr_workspace_bytes(256, 4096, 32768, 10)
    for bad in ((0, 4096, 100, 1), (1, 4095, 100, 1), (1, 4096, 0, 1), (1, 4096, 100, 0),
                (1, 4096, 100, 65), (1, 4096, 5, 6)):
        assert fr.fr_workspace_bytes(*bad) == 0


def _draft(H=0x1000, M=10, d=4096, W=0x2000, idx=0, V=32768, k=10, ids=0x3000, lp=0x4000,
           ws=0x5000, ws_bytes=1 << 26):
    return fr.lib().fr_draft_topk(H, M, d, W, idx, V, k, ids, lp, ws, ws_bytes, None)


def test_draft_topk_rejects_bad_arguments_before_any_launch():
    # the pointers are fake: reaching a kernel launch would be an error in itself
    assert _draft(H=0) == INVALID
    assert _draft(W=0) == INVALID
    assert _draft(ids=0) == INVALID
    assert _draft(lp=0) == INVALID
    assert _draft(ws=0) == INVALID
    assert _draft(M=0) == INVALID
    assert _draft(d=4100) == INVALID
    assert _draft(k=0) == INVALID
    assert _draft(k=65) == INVALID
    assert _draft(V=5, k=6) == INVALID
    assert _draft(V=1 << 20, d=4096) == UNSUPPORTED       # 8 GiB of weights: beyond the 32-bit offsets
    assert _draft(V=(1 << 19) + 1, d=4096) == UNSUPPORTED
    assert _draft(V=1 << 19, d=4096, ws_bytes=1024) == WORKSPACE   # exactly 4 GiB passes the shape check
    assert _draft(H=0x1008) == ALIGN
    assert _draft(W=0x2004) == ALIGN
    assert _draft(ws=0x5008) == ALIGN
    assert _draft(ws_bytes=1024) == WORKSPACE
    need = fr.fr_workspace_bytes(10, 4096, 32768, 10)
    assert _draft(ws_bytes=need - 1) == WORKSPACE


def test_full_topk_and_logits_reject_bad_arguments():
    L = fr.lib()
    assert L.fr_full_topk(0, 1, 64, 0x2000, 100, 1, 0x3000, 0x4000, 0x5000, 1 << 26, None) == INVALID
    assert L.fr_full_topk(0x1000, 1, 64, 0x2000, 100, 101, 0x3000, 0x4000, 0x5000, 1 << 26, None) == INVALID
    assert L.fr_draft_logits(0x1000, 1, 64, 0x2000, 100, 0, None) == INVALID
    assert L.fr_draft_logits(0x1001, 1, 64, 0x2000, 100, 0x3000, None) == ALIGN


def test_tuned_entry_validates_knobs():
    t = Tuning()
    t.path = 7
    st = fr.lib().fr_draft_topk_tuned(0x1000, 10, 4096, 0x2000, 0, 32768, 10, 0x3000, 0x4000,
                                      0x5000, 1 << 26, None, ctypes.byref(t))
    assert st == INVALID


def test_build_subset_rejects_bad_arguments():
    L = fr.lib()
    ok = dict(W=0x1000, V=100, d=64, ids=0x2000, Vs=10, Ws=0x3000, im=0x4000)

    def call(**kw):
        a = {**ok, **kw}
        return L.fr_build_subset(a["W"], a["V"], a["d"], a["ids"], a["Vs"], a["Ws"], a["im"], None, None)

    assert call(W=0) == INVALID and call(ids=0) == INVALID and call(Ws=0) == INVALID and call(im=0) == INVALID
    assert call(Vs=0) == INVALID and call(Vs=101) == INVALID and call(d=60) == INVALID and call(V=0) == INVALID
    assert call(W=0x1004) == ALIGN and call(Ws=0x3008) == ALIGN


def test_workspace_init_and_calib_reject_bad_arguments():
    L = fr.lib()
    assert L.fr_workspace_init(0, 4096, None) == INVALID
    assert L.fr_workspace_init(0x1000, 16, None) == WORKSPACE
    assert L.fr_calib_copy(0x1000, 0x2000, 24, None) == INVALID
    assert L.fr_calib_read(0, 1024, 0x1000, None) == INVALID


def test_binding_refuses_cpu_tensors():
    import torch
    H = torch.zeros((2, 64), dtype=torch.bfloat16)
    W = torch.zeros((8, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        fr.fr_draft_topk(H, W, None, 2, torch.zeros(1 << 20, dtype=torch.uint8))


def test_beam_glue_rejects_bad_arguments_before_any_launch():
    L = fr.lib()
    UNSUPPORTED = -5
    P = [0x1000 * (i + 1) for i in range(10)]

    def expand(logp=P[0], tok=P[1], M=10, k=10, ns=P[2], nh=P[3], width=10, hs=P[4], ht=P[5], hp=P[6], off=0,
               os_=P[7], ot=P[8], oh=P[9]):
        return L.fr_beam_expand(logp, tok, M, k, ns, nh, width, hs, ht, hp, off, os_, ot, oh, None)

    assert expand(logp=0) == INVALID and expand(oh=0) == INVALID and expand(hs=0) == INVALID
    assert expand(M=0) == INVALID and expand(k=0) == INVALID and expand(width=0) == INVALID
    assert expand(width=101) == INVALID and expand(off=-1) == INVALID
    assert expand(M=65, k=64) == UNSUPPORTED          # more than 4096 candidates in one step

    def select(hs=P[0], ht=P[1], hp=P[2], N=600, K=60, a=P[3], b=P[4], c=P[5], d=P[6], m=P[7]):
        return L.fr_tree_select(hs, ht, hp, N, K, a, b, c, d, m, None)

    assert select(hs=0) == INVALID and select(m=0) == INVALID
    assert select(N=0) == INVALID and select(K=0) == INVALID and select(N=50, K=60) == INVALID
    assert select(N=5000) == UNSUPPORTED and select(N=4096, K=2000) == UNSUPPORTED


def test_multi_block_entry_rejects_bad_arguments():
    L = fr.lib()
    two = (ctypes.c_void_p * 2)(0x1000, 0x9000)
    bad = (ctypes.c_void_p * 2)(0x1000, 0)
    odd = (ctypes.c_void_p * 2)(0x1000, 0x9008)

    def call(ptrs=two, n=2, rows=5, d=4096, W=0x20000, V=32768, k=10, ids=0x3000, lp=0x4000, ws=0x5000):
        return L.fr_draft_topk_multi(ptrs, n, rows, d, W, 0, V, k, ids, lp, ws, 1 << 26, None)

    assert call(ptrs=None) == INVALID and call(n=0) == INVALID and call(n=17) == INVALID
    assert call(rows=0) == INVALID and call(ptrs=bad) == INVALID and call(ptrs=odd) == ALIGN
    assert call(k=0) == INVALID and call(W=0) == INVALID and call(ids=0) == INVALID


def test_token_statistics_reject_bad_arguments():
    L = fr.lib()
    UNSUPPORTED = -5
    assert L.fr_count_tokens(0x1000, 10, 100, 0, None, None) == INVALID
    assert L.fr_count_tokens(0, 10, 100, 0x2000, None, None) == INVALID
    assert L.fr_count_tokens(0x1000, -1, 100, 0x2000, None, None) == INVALID
    assert L.fr_count_tokens(0x1000, 10, 0, 0x2000, None, None) == INVALID
    assert L.fr_count_tokens(0x1004, 10, 100, 0x2000, None, None) == ALIGN
    assert L.fr_count_tokens(0x1000, 10, 100, 0x2004, None, None) == ALIGN
    assert L.fr_count_tokens(0x1000, 0, 100, 0x2000, None, None) == 0          # nothing to do, nothing launched
    assert L.fr_count_tokens(0x1000, 10, (1 << 22) + 1, 0x2000, None, None) == UNSUPPORTED
    assert L.fr_rank_tokens(0, 100, 0x2000, None) == INVALID
    assert L.fr_rank_tokens(0x1000, 0, 0x2000, None) == INVALID
    assert L.fr_rank_tokens(0x1000, (1 << 22) + 1, 0x2000, None) == UNSUPPORTED


def test_draft_step_rejects_bad_arguments_before_any_launch():
    L = fr.lib()
    P = [0x1000 * (i + 1) for i in range(16)]

    def step(H=P[0], M=10, d=4096, W=P[1], V=32768, k=10, ns=P[2], nh=P[3], width=10, hs=P[4], ht=P[5], hp=P[6],
             off=0, ids=P[7], lp=P[8], os_=P[9], ot=P[10], oh=P[11], ws=P[12]):
        return L.fr_draft_step(H, M, d, W, 0, V, k, ns, nh, width, hs, ht, hp, off, ids, lp, os_, ot, oh, ws,
                               1 << 26, None)

    assert step(ns=0) == INVALID and step(oh=0) == INVALID and step(hs=0) == INVALID
    assert step(width=0) == INVALID and step(width=101) == INVALID and step(off=-1) == INVALID
    assert step(H=0) == INVALID and step(k=0) == INVALID and step(ids=0) == INVALID
