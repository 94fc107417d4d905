"""The C-ABI library loads without a GPU, exports every symbol the header declares, and
rejects host-checkable mistakes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2506_14158_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return B.lib()


def test_every_declared_symbol_is_exported(L):
    hdr = open(os.path.join(ROOT, "include", "s4c.h")).read()
    declared = set(re.findall(r"\b(s4c_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_strerror(L):
    assert B.s4c_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -6, -77):
        assert len(B.s4c_strerror(code)) > 0


def shape(**kw):
    d = dict(B=2, Hq=8, Hkv=2, D=128, N=64, S_cap=4096 + 64, dtype=B.S4C_BF16)
    d.update(kw)
    return B.AttnShape(**d)


def test_workspace_queries(L):
    s = shape()
    assert B.s4c_tree_attn_num_splits(s, 4096) >= 1
    n = B.s4c_tree_attn_workspace_size(s, 4096)
    assert n % 256 == 0
    assert B.s4c_tree_attn_workspace_size(shape(N=129), 4096) == 0
    assert B.s4c_tree_attn_workspace_size(shape(Hq=7), 4096) == 0
    assert B.s4c_accept_path_workspace_size(2, 64, 32000) > 0
    assert B.s4c_accept_path_workspace_size(0, 64, 32000) == 0
    # deterministic plan
    assert B.s4c_tree_attn_num_splits(s, 4096) == B.s4c_tree_attn_num_splits(shape(), 4096)


def test_tree_attn_host_errors(L):
    s = shape()
    one = C.c_void_p(256)          # never dereferenced: all of these fail before any launch
    call = lambda sh, q=one, ws=None, wsb=0, mcl=4096: L.s4c_tree_attn(
        C.byref(sh), q, one, one, one, one, one, one, mcl, 0.0, one, None, ws, wsb, None)
    assert call(s, q=None) == -1
    assert call(shape(N=200)) == -3
    assert call(shape(D=96)) == -3
    assert call(shape(dtype=7)) == -3
    assert call(shape(Hq=7)) == -2
    assert call(shape(B=0)) == -2
    assert call(s, mcl=10 ** 6) == -2                      # max_cache_len beyond S_cap
    assert call(s, q=C.c_void_p(264)) == -2                # Q / K / V / out must be 16-byte aligned
    if B.s4c_tree_attn_workspace_size(s, 4096) > 0:
        assert call(s) == -4                               # workspace required but missing
        assert call(s, ws=one, wsb=16) == -4


def test_accept_and_compact_host_errors(L):
    one = C.c_void_p(256)
    acc = lambda Bn=2, N=8, V=100, dt=1, mode=0, T=1.0, logits=one, pd=one, ws=one, wsb=1 << 20, mp=4: \
        L.s4c_accept_path(Bn, N, V, dt, mode, T, logits, one, one, pd, one, mp, one, one, one, one, None, ws, wsb, None)
    assert acc(logits=None) == -1
    assert acc(N=129) == -3
    assert acc(mode=5) == -3
    assert acc(dt=9) == -3
    assert acc(V=0) == -2
    assert acc(mp=0) == -2
    assert acc(mode=1, pd=None) == -1
    assert acc(mode=1, T=0.0) == -2
    assert acc(ws=None) == -4
    assert acc(wsb=8) == -4
    # the entry point without a workspace: same checks, and problems beyond its fixed scratch are refused
    st = lambda Bn=2, N=8, V=100, mode=0, logits=one, pd=one: \
        L.s4c_accept_path_static(Bn, N, V, 1, mode, 1.0, logits, one, one, pd, one, 4, one, one, one, one, None, None)
    assert st(logits=None) == -1 and st(N=129) == -3 and st(V=0) == -2 and st(mode=1, pd=None) == -1
    assert B.s4c_accept_path_workspace_size(16, 128, 2000000) > B.S4C_STATIC_SCRATCH_BYTES
    assert st(Bn=16, N=128, V=2000000) == -6 and "static scratch" in B.s4c_strerror(-6)
    s = shape()
    cmp_ = lambda sh=s, kt=one, mp=4: L.s4c_kv_compact(C.byref(sh), kt, one, one, one, one, one, one, mp, None, None, None)
    assert cmp_(kt=None) == -1
    assert cmp_(sh=shape(D=100)) == -3
    assert cmp_(mp=0) == -2


def test_paged_and_multi_layer_host_errors(L):
    """Every check below fails before any launch (no GPU needed): null pointers, page sizes that are not
    powers of two >= 64, a logical capacity that disagrees with the block table, layer counts."""
    one = C.c_void_p(256)
    s = shape(S_cap=64 * 128)
    pa = lambda sh=s, bt=one, mb=64, ps=128, npg=200: L.s4c_tree_attn_paged(
        C.byref(sh), one, one, one, one, one, bt, mb, ps, npg, one, one, 4096, 0.0, one, None, one, 1 << 30, None)
    assert pa(bt=None) == -1
    assert pa(ps=96) == -3 and pa(ps=32) == -3
    assert pa(mb=0) == -2 and pa(npg=0) == -2
    assert pa(mb=63) == -2                                   # S_cap != max_blocks * page_size
    cp = lambda sh=s, bt=one, mb=64, ps=128, npg=200, mp=4: L.s4c_kv_compact_paged(
        C.byref(sh), one, one, one, one, bt, mb, ps, npg, one, one, one, mp, None, None, None)
    assert cp(bt=None) == -1 and cp(ps=100) == -3 and cp(mb=0) == -2 and cp(mp=0) == -2
    cm = lambda sh=s, layers=4, kt=one, feats=None, fo=None, fb=0, mp=4: L.s4c_commit_path(
        C.byref(sh), layers, kt, one, one, one, one, one, one, mp, feats, fb, fo, None, None, None)
    assert cm(kt=None) == -1 and cm(layers=0) == -2 and cm(layers=70000) == -2 and cm(mp=0) == -2
    assert cm(feats=one, fo=None, fb=64) == -1               # features and features_out go together
    assert cm(feats=one, fo=one, fb=24) == -2                # rows must be multiples of 16 bytes
    cmp_ = lambda bt=one, ps=128, mb=64, npg=200, layers=4: L.s4c_commit_path_paged(
        C.byref(s), layers, one, one, one, one, bt, mb, ps, npg, one, one, one, 4, None, 0, None, None, None, None)
    assert cmp_(bt=None) == -1 and cmp_(ps=48) == -3 and cmp_(mb=0) == -2 and cmp_(layers=0) == -2
    dl = lambda T=300, H=64, Hout=256, dt=1, e=one, ws=None, wsb=0: L.s4c_draft_linear(T, H, Hout, dt, e, one, one, None, one,
                                                                                         ws, wsb, None)
    assert dl(e=None) == -1 and dl(T=0) == -2 and dl(dt=0) == -3 and dl(H=40) == -3 and dl(Hout=100) == -3
    assert dl(e=C.c_void_p(8)) == -2                          # 16-byte alignment
    # up to 512 tokens the call streams W (passes of at most 128 tokens) with split-K partial sums in a workspace
    assert B.s4c_draft_linear_workspace_size(600, 64, 256) == 0 and dl(T=600, e=C.c_void_p(16)) != -4
    assert B.s4c_draft_linear_workspace_size(300, 64, 256) >= 100 * 256 * 4 and dl(T=300) == -4
    need = B.s4c_draft_linear_workspace_size(60, 4096, 4096)
    assert need >= 60 * 4096 * 4 and need % 256 == 0
    assert dl(T=60, H=4096, Hout=4096) == -4 and dl(T=60, H=4096, Hout=4096, ws=one, wsb=need - 1) == -4


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libs4c.so")
    with pytest.raises(FileNotFoundError):
        B.lib()
