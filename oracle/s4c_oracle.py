"""ctypes wrapper of the CPU oracle (TEST INFRASTRUCTURE -- never used by the product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It compiles ``s4c_oracle.c`` with gcc on first use and marshals numpy arrays; all of the
arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s4c_oracle.c")
_LIB = os.path.join(_HERE, "libs4c_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "s4c_oracle.h"))):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "N", "S_cap", "dtype")]


def _load():
    global _lib
    if _lib is None:
        # S4C_ORACLE_LIB: a library somebody else built from the same source (the sanitizer test's
        # instrumented build); otherwise build in place if stale
        _lib = C.CDLL(os.environ.get("S4C_ORACLE_LIB") or build())
        for name in ("oracle_tree_attn", "oracle_tree_attn_sampled", "oracle_accept_path",
                     "oracle_row_stats", "oracle_kv_compact", "oracle_num_threads", "oracle_accept_resample", "oracle_commit_path", "oracle_build_tree", "oracle_draft_linear", "oracle_paged_gather", "oracle_kv_compact_paged", "oracle_decode", "oracle_commit_path_paged"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float16:
        return 2
    raise TypeError("oracle arrays must be float32, uint16 (bf16 bits) or float16, got %s" % a.dtype)


def decode(a: np.ndarray) -> np.ndarray:
    """Stored elements (float32 / bf16 bits as uint16 / float16) -> the doubles the oracle computes with."""
    a = np.ascontiguousarray(a)
    out = np.empty(a.size, dtype=np.float64)
    _load().oracle_decode(_dt(a), a.size, _p(a), _p(out))
    return out.reshape(a.shape)


def _p(a):
    if a is None:
        return C.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _shape(q, k_tree, k_cache):
    B, N, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    S_cap = k_cache.shape[2]
    assert k_tree.shape == (B, N, Hkv, D) and k_cache.shape == (B, Hkv, S_cap, D)
    return _Shape(B, Hq, Hkv, D, N, S_cap, _dt(q))


def tree_attn(q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, scale=0.0):
    """-> (out float64 [B][N][Hq][D], status int32 [B])"""
    lib = _load()
    s = _shape(q, k_tree, k_cache)
    cache_len, parent = _i32(cache_len), _i32(parent)
    out = np.empty(q.shape, dtype=np.float64)
    status = np.zeros(s.B, dtype=np.int32)
    rc = lib.oracle_tree_attn(C.byref(s), _p(q), _p(k_tree), _p(v_tree), _p(k_cache), _p(v_cache),
                              _p(cache_len), _p(parent), C.c_double(scale), _p(out), _p(status))
    assert rc == 0
    return out, status


def tree_attn_sampled(q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, bnh, scale=0.0):
    """bnh int32 [n][3] = (sequence, node, query head) -> out float64 [n][D]"""
    lib = _load()
    s = _shape(q, k_tree, k_cache)
    cache_len, parent, bnh = _i32(cache_len), _i32(parent), _i32(bnh)
    n = bnh.shape[0]
    out = np.empty((n, s.D), dtype=np.float64)
    rc = lib.oracle_tree_attn_sampled(C.byref(s), _p(q), _p(k_tree), _p(v_tree), _p(k_cache), _p(v_cache),
                                      _p(cache_len), _p(parent), C.c_double(scale), C.c_int32(n), _p(bnh), _p(out))
    assert rc == 0, rc
    return out


def row_stats(logits, temperature=1.0):
    """logits [rows][V] -> (argmax int32, max float64, sumexp float64)"""
    lib = _load()
    rows, V = logits.shape
    g = np.empty(rows, dtype=np.int32)
    m = np.empty(rows, dtype=np.float64)
    S = np.empty(rows, dtype=np.float64)
    rc = lib.oracle_row_stats(C.c_int32(rows), C.c_int32(V), C.c_int32(_dt(logits)), C.c_double(temperature),
                              _p(logits), _p(g), _p(m), _p(S))
    assert rc == 0
    return g, m, S


def accept_path(logits, parent, tokens, mode, max_path, p_draft=None, uniforms=None, temperature=1.0):
    """mode "greedy"|"stochastic" -> dict(path, accept_len, accepted_tokens, bonus_token, margin, status)"""
    lib = _load()
    B, N, V = logits.shape
    parent, tokens = _i32(parent), _i32(tokens)
    m = {"greedy": 0, "stochastic": 1}[mode]
    if m == 1:
        p_draft = np.ascontiguousarray(p_draft, dtype=np.float32)
        uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
    path = np.empty((B, max_path), dtype=np.int32)
    atok = np.empty((B, max_path), dtype=np.int32)
    alen = np.empty(B, dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    margin = np.empty(B, dtype=np.float64)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_accept_path(C.c_int32(B), C.c_int32(N), C.c_int32(V), C.c_int32(_dt(logits)), C.c_int32(m),
                                C.c_double(temperature), _p(logits), _p(parent), _p(tokens),
                                _p(p_draft if m == 1 else None), _p(uniforms if m == 1 else None),
                                C.c_int32(max_path), _p(path), _p(alen), _p(atok), _p(bonus), _p(margin), _p(status))
    assert rc == 0, rc
    return dict(path=path, accept_len=alen, accepted_tokens=atok, bonus_token=bonus, margin=margin, status=status)


def accept_resample(logits, draft_probs, parent, tokens, uniforms, u_resample, max_path, temperature=1.0):
    """Sibling-sequential rule with the correction token
    -> dict(path, accept_len, accepted_tokens, bonus_token, margin_accept, margin_sample, status)"""
    lib = _load()
    B, N, V = logits.shape
    parent, tokens = _i32(parent), _i32(tokens)
    draft_probs = np.ascontiguousarray(draft_probs, dtype=np.float32)
    assert draft_probs.shape == (B, N, V)
    uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
    u_resample = np.ascontiguousarray(u_resample, dtype=np.float32)
    assert uniforms.shape == (B, N) and u_resample.shape == (B,)
    path = np.empty((B, max_path), dtype=np.int32)
    atok = np.empty((B, max_path), dtype=np.int32)
    alen = np.empty(B, dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    ma = np.empty(B, dtype=np.float64)
    ms = np.empty(B, dtype=np.float64)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_accept_resample(C.c_int32(B), C.c_int32(N), C.c_int32(V), C.c_int32(_dt(logits)),
                                    C.c_double(temperature), _p(logits), _p(draft_probs), _p(parent), _p(tokens),
                                    _p(uniforms), _p(u_resample), C.c_int32(max_path), _p(path), _p(alen), _p(atok),
                                    _p(bonus), _p(ma), _p(ms), _p(status))
    assert rc == 0, rc
    return dict(path=path, accept_len=alen, accepted_tokens=atok, bonus_token=bonus, margin_accept=ma,
                margin_sample=ms, status=status)


def kv_compact(k_tree, v_tree, k_cache, v_cache, cache_len, path, accept_len):
    """In place on k_cache, v_cache, cache_len (numpy arrays) -> (dst_index, status)"""
    lib = _load()
    B, N, Hkv, D = k_tree.shape
    S_cap = k_cache.shape[2]
    s = _Shape(B, Hkv, Hkv, D, N, S_cap, _dt(k_tree))
    assert cache_len.dtype == np.int32 and cache_len.flags["C_CONTIGUOUS"]
    path, accept_len = _i32(path), _i32(accept_len)
    max_path = path.shape[1]
    dst = np.empty((B, max_path), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_kv_compact(C.byref(s), _p(k_tree), _p(v_tree), _p(k_cache), _p(v_cache), _p(cache_len),
                               _p(path), _p(accept_len), C.c_int32(max_path), _p(dst), _p(status))
    assert rc == 0
    return dst, status


def commit_path(k_tree, v_tree, k_cache, v_cache, cache_len, path, accept_len, features=None, features_out=None):
    """Multi-layer compaction, in place on k_cache, v_cache [layers][B][Hkv][S_cap][D], cache_len and
    features_out ([B][max_path][F], any dtype) -> (dst_index, status)"""
    lib = _load()
    Ly, B, N, Hkv, D = k_tree.shape
    S_cap = k_cache.shape[3]
    assert k_cache.shape == (Ly, B, Hkv, S_cap, D) and v_tree.shape == k_tree.shape and v_cache.shape == k_cache.shape
    s = _Shape(B, Hkv, Hkv, D, N, S_cap, _dt(k_tree))
    assert cache_len.dtype == np.int32 and cache_len.flags["C_CONTIGUOUS"]
    path, accept_len = _i32(path), _i32(accept_len)
    max_path = path.shape[1]
    fb = 0
    if features is not None:
        assert features.shape[:2] == (B, N) and features_out.shape[:2] == (B, max_path)
        fb = int(features[0, 0].nbytes)
        assert int(features_out[0, 0].nbytes) == fb
    dst = np.empty((B, max_path), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_commit_path(C.byref(s), C.c_int32(Ly), _p(k_tree), _p(v_tree), _p(k_cache), _p(v_cache),
                                _p(cache_len), _p(path), _p(accept_len), C.c_int32(max_path), _p(features),
                                C.c_int32(fb), _p(features_out), _p(dst), _p(status))
    assert rc == 0
    return dst, status


def build_tree(draft_logits, nchild, root_token, kmax, temperature=1.0):
    """draft_logits [B][N][V], nchild [B][N] -> dict(parent, tokens, p_draft, level, status)"""
    lib = _load()
    B, N, V = draft_logits.shape
    nchild, root_token = _i32(nchild), _i32(root_token)
    assert nchild.shape == (B, N) and root_token.shape == (B,)
    parent = np.empty((B, N), dtype=np.int32)
    tokens = np.empty((B, N), dtype=np.int32)
    pd = np.empty((B, N), dtype=np.float32)
    level = np.empty((B, N), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_build_tree(C.c_int32(B), C.c_int32(N), C.c_int32(V), C.c_int32(_dt(draft_logits)),
                               C.c_double(temperature), _p(draft_logits), _p(nchild), _p(root_token), C.c_int32(kmax),
                               _p(parent), _p(tokens), _p(pd), _p(level), _p(status))
    assert rc == 0, rc
    return dict(parent=parent, tokens=tokens, p_draft=pd, level=level, status=status)


def draft_linear(e, f, W, bias=None):
    """e, f [T][H], W [Hout][2H], bias [Hout] or None -> out float64 [T][Hout]"""
    lib = _load()
    T, H = e.shape
    Hout = W.shape[0]
    assert f.shape == (T, H) and W.shape == (Hout, 2 * H) and _dt(e) == _dt(f) == _dt(W)
    assert bias is None or (bias.shape == (Hout,) and _dt(bias) == _dt(e))
    out = np.empty((T, Hout), dtype=np.float64)
    rc = lib.oracle_draft_linear(C.c_int32(T), C.c_int32(H), C.c_int32(Hout), C.c_int32(_dt(e)), _p(e), _p(f), _p(W),
                                 _p(bias), _p(out))
    assert rc == 0
    return out


def paged_gather(pool, block_table, cache_len, S_cap):
    """pool [num_pages][Hkv][page_size][D], block_table [B][max_blocks] -> (cache [B][Hkv][S_cap][D], status)"""
    lib = _load()
    num_pages, Hkv, page_size, D = pool.shape
    block_table, cache_len = _i32(block_table), _i32(cache_len)
    B, max_blocks = block_table.shape
    s = _Shape(B, Hkv, Hkv, D, 1, S_cap, _dt(pool))
    cache = np.empty((B, Hkv, S_cap, D), dtype=pool.dtype)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_paged_gather(C.byref(s), C.c_int32(page_size), C.c_int32(num_pages), C.c_int32(max_blocks), _p(pool),
                                 _p(block_table), _p(cache_len), _p(cache), _p(status))
    assert rc == 0
    return cache, status


def kv_compact_paged(k_tree, v_tree, k_pool, v_pool, block_table, cache_len, path, accept_len):
    """In place on k_pool, v_pool, cache_len -> (dst_index, status)"""
    lib = _load()
    B, N, Hkv, D = k_tree.shape
    num_pages, _, page_size, _ = k_pool.shape
    block_table = _i32(block_table)
    max_blocks = block_table.shape[1]
    s = _Shape(B, Hkv, Hkv, D, N, max_blocks * page_size, _dt(k_tree))
    assert cache_len.dtype == np.int32 and cache_len.flags["C_CONTIGUOUS"]
    path, accept_len = _i32(path), _i32(accept_len)
    max_path = path.shape[1]
    dst = np.empty((B, max_path), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_kv_compact_paged(C.byref(s), C.c_int32(page_size), C.c_int32(num_pages), C.c_int32(max_blocks),
                                     _p(k_tree), _p(v_tree), _p(k_pool), _p(v_pool), _p(block_table), _p(cache_len),
                                     _p(path), _p(accept_len), C.c_int32(max_path), _p(dst), _p(status))
    assert rc == 0
    return dst, status


def commit_path_paged(k_tree, v_tree, k_pool, v_pool, block_table, cache_len, path, accept_len, features=None,
                      features_out=None):
    """Multi-layer compaction into paged pools [layers][num_pages][Hkv][page][D] (one block table for all
    layers), in place on the pools, cache_len and features_out -> (dst_index, status)"""
    lib = _load()
    Ly, B, N, Hkv, D = k_tree.shape
    _, num_pages, _, page_size, _ = k_pool.shape
    assert k_pool.shape == (Ly, num_pages, Hkv, page_size, D) and v_pool.shape == k_pool.shape and v_tree.shape == k_tree.shape
    block_table = _i32(block_table)
    max_blocks = block_table.shape[1]
    s = _Shape(B, Hkv, Hkv, D, N, max_blocks * page_size, _dt(k_tree))
    assert cache_len.dtype == np.int32 and cache_len.flags["C_CONTIGUOUS"]
    path, accept_len = _i32(path), _i32(accept_len)
    max_path = path.shape[1]
    fb = 0
    if features is not None:
        assert features.shape[:2] == (B, N) and features_out.shape[:2] == (B, max_path)
        fb = int(features[0, 0].nbytes)
        assert int(features_out[0, 0].nbytes) == fb
    dst = np.empty((B, max_path), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib.oracle_commit_path_paged(C.byref(s), C.c_int32(Ly), C.c_int32(page_size), C.c_int32(num_pages),
                                      C.c_int32(max_blocks), _p(k_tree), _p(v_tree), _p(k_pool), _p(v_pool), _p(block_table),
                                      _p(cache_len), _p(path), _p(accept_len), C.c_int32(max_path), _p(features),
                                      C.c_int32(fb), _p(features_out), _p(dst), _p(status))
    assert rc == 0
    return dst, status
