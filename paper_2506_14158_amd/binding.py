"""Thin ctypes binding of libs4c.so: same names as the C ABI, argument marshalling only.

Every step of the tree-verification path runs in the HIP kernels behind these calls; PyTorch
supplies device memory and the stream.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libs4c.so")

S4C_F32, S4C_BF16, S4C_F16 = 0, 1, 2
S4C_GREEDY, S4C_STOCHASTIC = 0, 1
S4C_SEQ_BAD_TREE, S4C_SEQ_BAD_LEN, S4C_SEQ_TIMEOUT = 1, 2, 4

EXPORTS = ("s4c_tree_attn_workspace_size", "s4c_tree_attn", "s4c_accept_path_workspace_size",
           "s4c_accept_path", "s4c_kv_compact", "s4c_strerror", "s4c_tree_attn_num_splits",
           "s4c_accept_resample", "s4c_accept_resample_workspace_size", "s4c_commit_path", "s4c_build_tree", "s4c_build_tree_workspace_size",
           "s4c_draft_linear", "s4c_draft_linear_workspace_size", "s4c_tree_attn_paged", "s4c_kv_compact_paged", "s4c_commit_path_paged", "s4c_accept_path_static")


class S4CError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libs4c: %s (status %d)" % (msg, code))
        self.code = code


class AttnShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "N", "S_cap", "dtype")]


_lib = None


def lib() -> C.CDLL:
    """Load libs4c.so (built in-tree by ``__graft_entry__.build()``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build the HIP library first (python -c 'import __graft_entry__ as g; g.build()')"
                % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.s4c_tree_attn_workspace_size.restype = C.c_size_t
        L.s4c_tree_attn_workspace_size.argtypes = [C.POINTER(AttnShape), C.c_int32]
        L.s4c_tree_attn_num_splits.restype = C.c_int32
        L.s4c_tree_attn_num_splits.argtypes = [C.POINTER(AttnShape), C.c_int32]
        L.s4c_tree_attn.restype = C.c_int
        L.s4c_tree_attn.argtypes = [C.POINTER(AttnShape)] + [C.c_void_p] * 7 + [
            C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.s4c_accept_path_workspace_size.restype = C.c_size_t
        L.s4c_accept_path_workspace_size.argtypes = [C.c_int32] * 3
        L.s4c_accept_path.restype = C.c_int
        L.s4c_accept_path.argtypes = [C.c_int32] * 5 + [C.c_float] + [C.c_void_p] * 5 + [C.c_int32] + [
            C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        L.s4c_accept_resample.restype = C.c_int
        L.s4c_accept_resample.argtypes = [C.c_int32] * 4 + [C.c_float] + [C.c_void_p] * 6 + [C.c_int32] + [
            C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        L.s4c_accept_resample_workspace_size.restype = C.c_size_t
        L.s4c_accept_resample_workspace_size.argtypes = [C.c_int32] * 4
        L.s4c_kv_compact.restype = C.c_int
        L.s4c_kv_compact.argtypes = [C.POINTER(AttnShape)] + [C.c_void_p] * 7 + [C.c_int32] + [C.c_void_p] * 3
        L.s4c_commit_path.restype = C.c_int
        L.s4c_commit_path.argtypes = [C.POINTER(AttnShape), C.c_int32] + [C.c_void_p] * 7 + [C.c_int32, C.c_void_p,
                                                                                          C.c_int32] + [C.c_void_p] * 4
        L.s4c_commit_path_paged.restype = C.c_int
        L.s4c_commit_path_paged.argtypes = [C.POINTER(AttnShape), C.c_int32] + [C.c_void_p] * 5 + [C.c_int32] * 3 + \
            [C.c_void_p] * 3 + [C.c_int32, C.c_void_p, C.c_int32] + [C.c_void_p] * 4
        L.s4c_build_tree_workspace_size.restype = C.c_size_t
        L.s4c_build_tree_workspace_size.argtypes = [C.c_int32] * 3
        L.s4c_build_tree.restype = C.c_int
        L.s4c_build_tree.argtypes = [C.c_int32] * 4 + [C.c_float] + [C.c_void_p] * 3 + [C.c_int32] + [
            C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        L.s4c_tree_attn_paged.restype = C.c_int
        L.s4c_tree_attn_paged.argtypes = [C.POINTER(AttnShape)] + [C.c_void_p] * 6 + [C.c_int32] * 3 + [C.c_void_p] * 2 + [
            C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.s4c_kv_compact_paged.restype = C.c_int
        L.s4c_kv_compact_paged.argtypes = [C.POINTER(AttnShape)] + [C.c_void_p] * 5 + [C.c_int32] * 3 + [C.c_void_p] * 3 + [
            C.c_int32] + [C.c_void_p] * 3
        L.s4c_draft_linear.restype = C.c_int
        L.s4c_draft_linear.argtypes = [C.c_int32] * 4 + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        L.s4c_draft_linear_workspace_size.restype = C.c_size_t
        L.s4c_draft_linear_workspace_size.argtypes = [C.c_int32] * 3
        L.s4c_accept_path_static.restype = C.c_int
        L.s4c_accept_path_static.argtypes = [C.c_int32] * 5 + [C.c_float] + [C.c_void_p] * 5 + [C.c_int32] + [
            C.c_void_p] * 6
        L.s4c_strerror.restype = C.c_char_p
        L.s4c_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def s4c_strerror(code: int) -> str:
    return lib().s4c_strerror(code).decode()


def _check(code: int):
    if code != 0:
        raise S4CError(code, s4c_strerror(code))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libs4c takes contiguous device tensors")
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return S4C_F32
    if t.dtype == torch.bfloat16:
        return S4C_BF16
    if t.dtype == torch.float16:
        return S4C_F16
    raise TypeError("libs4c supports float32, bfloat16 and float16, got %s" % t.dtype)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def attn_shape(q: torch.Tensor, k_tree: torch.Tensor, k_cache: torch.Tensor) -> AttnShape:
    B, N, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    S_cap = k_cache.shape[2]
    if tuple(k_tree.shape) != (B, N, Hkv, D) or tuple(k_cache.shape) != (B, Hkv, S_cap, D):
        raise ValueError("inconsistent q / k_tree / k_cache shapes")
    return AttnShape(B, Hq, Hkv, D, N, S_cap, _dtype_code(q))


def s4c_tree_attn_workspace_size(shape: AttnShape, max_cache_len: int) -> int:
    return int(lib().s4c_tree_attn_workspace_size(C.byref(shape), max_cache_len))


def s4c_tree_attn_num_splits(shape: AttnShape, max_cache_len: int) -> int:
    return int(lib().s4c_tree_attn_num_splits(C.byref(shape), max_cache_len))


def s4c_tree_attn(q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, max_cache_len: int,
                  out: torch.Tensor, scale: float = 0.0, status: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Tree-masked attention of all N nodes; writes and returns ``out`` ([B][N][Hq][D])."""
    shape = attn_shape(q, k_tree, k_cache)
    for t in (k_tree, v_tree, k_cache, v_cache, out):
        if t.dtype != q.dtype:
            raise TypeError("q/k/v/cache/out must share one dtype")
    if v_tree.shape != k_tree.shape or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent v / out shapes")
    if cache_len.dtype != torch.int32 or parent.dtype != torch.int32 or tuple(parent.shape) != (shape.B, shape.N):
        raise TypeError("cache_len [B] and parent [B][N] must be int32")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().s4c_tree_attn(C.byref(shape), _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache),
                               _ptr(cache_len), _ptr(parent), int(max_cache_len), float(scale), _ptr(out),
                               _ptr(status), _ptr(workspace), ws_bytes, _stream()))
    return out


def s4c_tree_attn_paged(q, k_tree, v_tree, k_pool, v_pool, block_table, cache_len, parent, max_cache_len: int,
                        out: torch.Tensor, scale: float = 0.0, status: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Tree-masked attention over a paged cache: pools [num_pages][Hkv][page_size][D], block_table [B][max_blocks]."""
    B, N, Hq, D = q.shape
    num_pages, Hkv, page_size, _ = k_pool.shape
    max_blocks = int(block_table.shape[1])
    if tuple(k_tree.shape) != (B, N, Hkv, D) or v_tree.shape != k_tree.shape or v_pool.shape != k_pool.shape or \
            k_pool.shape[3] != D or out.shape != q.shape or tuple(block_table.shape) != (B, max_blocks):
        raise ValueError("inconsistent shapes")
    for t in (k_tree, v_tree, k_pool, v_pool, out):
        if t.dtype != q.dtype:
            raise TypeError("q/k/v/pools/out must share one dtype")
    for t in (block_table, cache_len, parent):
        if t.dtype != torch.int32:
            raise TypeError("block_table / cache_len / parent must be int32")
    shape = AttnShape(B, Hq, Hkv, D, N, max_blocks * page_size, _dtype_code(q))
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().s4c_tree_attn_paged(C.byref(shape), _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(k_pool), _ptr(v_pool),
                                     _ptr(block_table), max_blocks, int(page_size), int(num_pages), _ptr(cache_len),
                                     _ptr(parent), int(max_cache_len), float(scale), _ptr(out), _ptr(status),
                                     _ptr(workspace), ws_bytes, _stream()))
    return out


def s4c_kv_compact_paged(k_tree, v_tree, k_pool, v_pool, block_table, cache_len, path, accept_len,
                         dst_index: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    B, N, Hkv, D = k_tree.shape
    num_pages, _, page_size, _ = k_pool.shape
    max_blocks = int(block_table.shape[1])
    if tuple(k_pool.shape) != (num_pages, Hkv, page_size, D) or v_tree.shape != k_tree.shape or v_pool.shape != k_pool.shape:
        raise ValueError("inconsistent shapes")
    for t in (block_table, cache_len, path, accept_len):
        if t.dtype != torch.int32:
            raise TypeError("block_table / cache_len / path / accept_len must be int32")
    shape = AttnShape(B, Hkv, Hkv, D, N, max_blocks * page_size, _dtype_code(k_tree))
    _check(lib().s4c_kv_compact_paged(C.byref(shape), _ptr(k_tree), _ptr(v_tree), _ptr(k_pool), _ptr(v_pool),
                                      _ptr(block_table), max_blocks, int(page_size), int(num_pages), _ptr(cache_len),
                                      _ptr(path), _ptr(accept_len), int(path.shape[1]), _ptr(dst_index), _ptr(status),
                                      _stream()))


def s4c_accept_path_workspace_size(B: int, N: int, V: int) -> int:
    return int(lib().s4c_accept_path_workspace_size(B, N, V))


def _accept_checks(logits, parent, tokens, max_path, path, accept_len, accepted_tokens, bonus_token, p_draft, uniforms):
    B, N, V = logits.shape
    for t in (parent, tokens):
        if t.dtype != torch.int32 or tuple(t.shape) != (B, N):
            raise TypeError("parent / tokens must be int32 [B][N]")
    if tuple(path.shape) != (B, max_path) or tuple(accepted_tokens.shape) != (B, max_path):
        raise ValueError("path / accepted_tokens must be [B][max_path]")
    for t in (path, accept_len, accepted_tokens, bonus_token):
        if t.dtype != torch.int32:
            raise TypeError("outputs must be int32")
    for t in (p_draft, uniforms):
        if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != (B, N)):
            raise TypeError("p_draft / uniforms must be float32 [B][N]")
    return B, N, V


def s4c_accept_path(logits, parent, tokens, mode: int, max_path: int, path, accept_len, accepted_tokens,
                    bonus_token, workspace, p_draft=None, uniforms=None, temperature: float = 1.0,
                    status: Optional[torch.Tensor] = None) -> None:
    B, N, V = _accept_checks(logits, parent, tokens, max_path, path, accept_len, accepted_tokens, bonus_token, p_draft, uniforms)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().s4c_accept_path(B, N, V, _dtype_code(logits), int(mode), float(temperature), _ptr(logits),
                                 _ptr(parent), _ptr(tokens), _ptr(p_draft), _ptr(uniforms), int(max_path),
                                 _ptr(path), _ptr(accept_len), _ptr(accepted_tokens), _ptr(bonus_token),
                                 _ptr(status), _ptr(workspace), ws_bytes, _stream()))


S4C_STATIC_SCRATCH_BYTES = 1 << 20


def s4c_accept_path_static(logits, parent, tokens, mode: int, max_path: int, path, accept_len, accepted_tokens,
                           bonus_token, p_draft=None, uniforms=None, temperature: float = 1.0,
                           status: Optional[torch.Tensor] = None) -> None:
    """s4c_accept_path without a workspace argument: the library's fixed per-GPU scratch is used."""
    B, N, V = _accept_checks(logits, parent, tokens, max_path, path, accept_len, accepted_tokens, bonus_token, p_draft, uniforms)
    _check(lib().s4c_accept_path_static(B, N, V, _dtype_code(logits), int(mode), float(temperature), _ptr(logits),
                                        _ptr(parent), _ptr(tokens), _ptr(p_draft), _ptr(uniforms), int(max_path),
                                        _ptr(path), _ptr(accept_len), _ptr(accepted_tokens), _ptr(bonus_token),
                                        _ptr(status), _stream()))


def s4c_accept_resample_workspace_size(B: int, N: int, V: int, max_path: int) -> int:
    return int(lib().s4c_accept_resample_workspace_size(B, N, V, max_path))


def s4c_accept_resample(logits, draft_probs, parent, tokens, uniforms, u_resample, max_path: int, path,
                        accept_len, accepted_tokens, bonus_token, workspace=None, temperature: float = 1.0,
                        status: Optional[torch.Tensor] = None) -> None:
    B, N, V = logits.shape
    for t in (parent, tokens):
        if t.dtype != torch.int32 or tuple(t.shape) != (B, N):
            raise TypeError("parent / tokens must be int32 [B][N]")
    if draft_probs.dtype != torch.float32 or tuple(draft_probs.shape) != (B, N, V):
        raise TypeError("draft_probs must be float32 [B][N][V]")
    if uniforms.dtype != torch.float32 or tuple(uniforms.shape) != (B, N):
        raise TypeError("uniforms must be float32 [B][N]")
    if u_resample.dtype != torch.float32 or tuple(u_resample.shape) != (B,):
        raise TypeError("u_resample must be float32 [B]")
    if tuple(path.shape) != (B, max_path) or tuple(accepted_tokens.shape) != (B, max_path):
        raise ValueError("path / accepted_tokens must be [B][max_path]")
    for t in (path, accept_len, accepted_tokens, bonus_token):
        if t.dtype != torch.int32:
            raise TypeError("outputs must be int32")
    _check(lib().s4c_accept_resample(B, N, V, _dtype_code(logits), float(temperature), _ptr(logits), _ptr(draft_probs),
                                     _ptr(parent), _ptr(tokens), _ptr(uniforms), _ptr(u_resample), int(max_path),
                                     _ptr(path), _ptr(accept_len), _ptr(accepted_tokens), _ptr(bonus_token),
                                     _ptr(status), _ptr(workspace),
                                     workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                     _stream()))


def s4c_kv_compact(k_tree, v_tree, k_cache, v_cache, cache_len, path, accept_len,
                   dst_index: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    B, N, Hkv, D = k_tree.shape
    S_cap = k_cache.shape[2]
    if tuple(k_cache.shape) != (B, Hkv, S_cap, D) or v_tree.shape != k_tree.shape or v_cache.shape != k_cache.shape:
        raise ValueError("inconsistent shapes")
    if cache_len.dtype != torch.int32 or path.dtype != torch.int32 or accept_len.dtype != torch.int32:
        raise TypeError("cache_len / path / accept_len must be int32")
    shape = AttnShape(B, Hkv, Hkv, D, N, S_cap, _dtype_code(k_tree))
    _check(lib().s4c_kv_compact(C.byref(shape), _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache),
                                _ptr(cache_len), _ptr(path), _ptr(accept_len), int(path.shape[1]),
                                _ptr(dst_index), _ptr(status), _stream()))


def s4c_commit_path(k_tree, v_tree, k_cache, v_cache, cache_len, path, accept_len, features=None, features_out=None,
                    dst_index: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    """k_tree/v_tree [layers][B][N][Hkv][D], caches [layers][B][Hkv][S_cap][D]; features [B][N][F] -> features_out
    [B][max_path][F] (same dtype)."""
    Ly, B, N, Hkv, D = k_tree.shape
    S_cap = k_cache.shape[3]
    if tuple(k_cache.shape) != (Ly, B, Hkv, S_cap, D) or v_tree.shape != k_tree.shape or v_cache.shape != k_cache.shape:
        raise ValueError("inconsistent shapes")
    if cache_len.dtype != torch.int32 or path.dtype != torch.int32 or accept_len.dtype != torch.int32:
        raise TypeError("cache_len / path / accept_len must be int32")
    max_path = int(path.shape[1])
    fb = 0
    if features is not None or features_out is not None:
        if features is None or features_out is None or features.dtype != features_out.dtype:
            raise TypeError("features and features_out go together and share a dtype")
        if tuple(features.shape[:2]) != (B, N) or tuple(features_out.shape[:2]) != (B, max_path) or \
                features.shape[2:] != features_out.shape[2:]:
            raise ValueError("features [B][N][F] / features_out [B][max_path][F]")
        fb = int(features[0, 0].numel() * features.element_size())
    shape = AttnShape(B, Hkv, Hkv, D, N, S_cap, _dtype_code(k_tree))
    _check(lib().s4c_commit_path(C.byref(shape), int(Ly), _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache),
                                 _ptr(cache_len), _ptr(path), _ptr(accept_len), max_path, _ptr(features), fb,
                                 _ptr(features_out), _ptr(dst_index), _ptr(status), _stream()))


def s4c_commit_path_paged(k_tree, v_tree, k_pool, v_pool, block_table, cache_len, path, accept_len, features=None,
                          features_out=None, dst_index: Optional[torch.Tensor] = None,
                          status: Optional[torch.Tensor] = None) -> None:
    """k_tree/v_tree [layers][B][N][Hkv][D], pools [layers][num_pages][Hkv][page][D], block_table [B][max_blocks]
    (one table for every layer); features as in s4c_commit_path."""
    Ly, B, N, Hkv, D = k_tree.shape
    _, num_pages, _, page, _ = k_pool.shape
    if tuple(k_pool.shape) != (Ly, num_pages, Hkv, page, D) or v_tree.shape != k_tree.shape or v_pool.shape != k_pool.shape:
        raise ValueError("inconsistent shapes")
    if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != B:
        raise TypeError("block_table must be int32 [B][max_blocks]")
    if cache_len.dtype != torch.int32 or path.dtype != torch.int32 or accept_len.dtype != torch.int32:
        raise TypeError("cache_len / path / accept_len must be int32")
    max_path, max_blocks = int(path.shape[1]), int(block_table.shape[1])
    fb = 0
    if features is not None or features_out is not None:
        if features is None or features_out is None or features.dtype != features_out.dtype:
            raise TypeError("features and features_out go together and share a dtype")
        if tuple(features.shape[:2]) != (B, N) or tuple(features_out.shape[:2]) != (B, max_path) or \
                features.shape[2:] != features_out.shape[2:]:
            raise ValueError("features [B][N][F] / features_out [B][max_path][F]")
        fb = int(features[0, 0].numel() * features.element_size())
    shape = AttnShape(B, Hkv, Hkv, D, N, max_blocks * page, _dtype_code(k_tree))
    _check(lib().s4c_commit_path_paged(C.byref(shape), int(Ly), _ptr(k_tree), _ptr(v_tree), _ptr(k_pool), _ptr(v_pool),
                                       _ptr(block_table), max_blocks, int(page), int(num_pages), _ptr(cache_len),
                                       _ptr(path), _ptr(accept_len), max_path, _ptr(features), fb, _ptr(features_out),
                                       _ptr(dst_index), _ptr(status), _stream()))


def s4c_build_tree_workspace_size(B: int, N: int, V: int) -> int:
    return int(lib().s4c_build_tree_workspace_size(B, N, V))


def s4c_build_tree(draft_logits, nchild, root_token, kmax: int, parent, tokens, p_draft, workspace,
                   temperature: float = 1.0, level: Optional[torch.Tensor] = None,
                   status: Optional[torch.Tensor] = None) -> None:
    B, N, V = draft_logits.shape
    for t in (nchild, parent, tokens) + ((level,) if level is not None else ()):
        if t.dtype != torch.int32 or tuple(t.shape) != (B, N):
            raise TypeError("nchild / parent / tokens / level must be int32 [B][N]")
    if root_token.dtype != torch.int32 or tuple(root_token.shape) != (B,):
        raise TypeError("root_token must be int32 [B]")
    if p_draft.dtype != torch.float32 or tuple(p_draft.shape) != (B, N):
        raise TypeError("p_draft must be float32 [B][N]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().s4c_build_tree(B, N, V, _dtype_code(draft_logits), float(temperature), _ptr(draft_logits),
                                _ptr(nchild), _ptr(root_token), int(kmax), _ptr(parent), _ptr(tokens), _ptr(p_draft),
                                _ptr(level), _ptr(status), _ptr(workspace), ws_bytes, _stream()))


def s4c_draft_linear_workspace_size(T: int, H: int, Hout: int) -> int:
    return int(lib().s4c_draft_linear_workspace_size(T, H, Hout))


def s4c_draft_linear(e, f, W, out, bias=None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[t] = W @ concat(e[t], f[t]) + bias (bf16 or fp16, fp32 accumulate); returns ``out``.  Up to 512 tokens
    the call needs ``workspace`` (s4c_draft_linear_workspace_size bytes)."""
    T, H = e.shape
    Hout = W.shape[0]
    if tuple(f.shape) != (T, H) or tuple(W.shape) != (Hout, 2 * H) or tuple(out.shape) != (T, Hout):
        raise ValueError("e, f [T][H]; W [Hout][2H]; out [T][Hout]")
    if bias is not None and tuple(bias.shape) != (Hout,):
        raise ValueError("bias [Hout]")
    for t in (e, f, W, out) + ((bias,) if bias is not None else ()):
        if t.dtype != e.dtype or e.dtype not in (torch.bfloat16, torch.float16):
            raise TypeError("s4c_draft_linear takes bfloat16 or float16 tensors of one type")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().s4c_draft_linear(T, H, Hout, _dtype_code(e), _ptr(e), _ptr(f), _ptr(W), _ptr(bias), _ptr(out),
                                  _ptr(workspace), ws_bytes, _stream()))
    return out


def alloc_workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    """Device scratch of at least nbytes (256-byte aligned by the torch allocator)."""
    if nbytes <= 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)
