"""One tree-verification step on the GPU: buffers + the three library calls, nothing else."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as _b


class TreeVerifier:
    """Pre-allocates outputs and workspaces for one shape and enqueues
    s4c_tree_attn -> s4c_accept_path -> s4c_kv_compact on the current stream."""

    def __init__(self, B, N, Hq, Hkv, D, S_cap, V, dtype: torch.dtype, max_path: int, max_cache_len: int,
                 device="cuda"):
        self.B, self.N, self.Hq, self.Hkv, self.D, self.S_cap, self.V = B, N, Hq, Hkv, D, S_cap, V
        self.dtype, self.max_path, self.max_cache_len = dtype, max_path, max_cache_len
        code = {torch.float32: _b.S4C_F32, torch.bfloat16: _b.S4C_BF16, torch.float16: _b.S4C_F16}[dtype]
        self.shape = _b.AttnShape(B, Hq, Hkv, D, N, S_cap, code)
        i32 = dict(dtype=torch.int32, device=device)
        self.out = torch.empty(B, N, Hq, D, dtype=dtype, device=device)
        self.attn_status = torch.zeros(B, **i32)
        self.path = torch.empty(B, max_path, **i32)
        self.accept_len = torch.empty(B, **i32)
        self.accepted_tokens = torch.empty(B, max_path, **i32)
        self.bonus_token = torch.empty(B, **i32)
        self.accept_status = torch.zeros(B, **i32)
        self.dst_index = torch.empty(B, max_path, **i32)
        self.compact_status = torch.zeros(B, **i32)
        self.attn_ws = _b.alloc_workspace(_b.s4c_tree_attn_workspace_size(self.shape, max_cache_len), device)
        self.accept_ws = _b.alloc_workspace(_b.s4c_accept_path_workspace_size(B, N, V), device)
        # sequential acceptance: the exchange slots of the workgroup teams (a few hundred KB at most), allocated
        # here so that no call allocates later (a step may be under graph capture)
        self.resample_ws = _b.alloc_workspace(max(256, _b.s4c_accept_resample_workspace_size(B, N, V, max_path)), device)
        self.num_splits = _b.s4c_tree_attn_num_splits(self.shape, max_cache_len)

    def tree_attn(self, q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, scale: float = 0.0):
        return _b.s4c_tree_attn(q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, self.max_cache_len,
                                self.out, scale, self.attn_status, self.attn_ws)

    def accept_path(self, logits, parent, tokens, mode: int, p_draft=None, uniforms=None, temperature=1.0):
        _b.s4c_accept_path(logits, parent, tokens, mode, self.max_path, self.path, self.accept_len,
                           self.accepted_tokens, self.bonus_token, self.accept_ws, p_draft, uniforms,
                           temperature, self.accept_status)

    def accept_resample(self, logits, draft_probs, parent, tokens, uniforms, u_resample, temperature=1.0):
        """Sibling-sequential rule with the correction token; same outputs as accept_path."""
        _b.s4c_accept_resample(logits, draft_probs, parent, tokens, uniforms, u_resample, self.max_path, self.path,
                               self.accept_len, self.accepted_tokens, self.bonus_token, self.resample_ws, temperature,
                               self.accept_status)

    def kv_compact(self, k_tree, v_tree, k_cache, v_cache, cache_len):
        _b.s4c_kv_compact(k_tree, v_tree, k_cache, v_cache, cache_len, self.path, self.accept_len,
                          self.dst_index, self.compact_status)

    def commit_path(self, k_tree, v_tree, k_cache, v_cache, cache_len, features=None, features_out=None):
        """All layers' K/V rows (leading [layers] dimension) and the feature rows of the accepted path."""
        _b.s4c_commit_path(k_tree, v_tree, k_cache, v_cache, cache_len, self.path, self.accept_len, features,
                           features_out, self.dst_index, self.compact_status)

    def step(self, q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, logits, tokens, mode: int,
             p_draft=None, uniforms=None, temperature: float = 1.0, scale: float = 0.0):
        self.tree_attn(q, k_tree, v_tree, k_cache, v_cache, cache_len, parent, scale)
        self.accept_path(logits, parent, tokens, mode, p_draft, uniforms, temperature)
        self.kv_compact(k_tree, v_tree, k_cache, v_cache, cache_len)
