"""Seeded synthetic tree-verification workloads.

This module only *draws inputs*: draft trees, per-node tokens, Q/K/V, the prefix
KV cache, target logits, draft probabilities and the uniform stream.  It holds
none of the method's arithmetic (no tree mask, no attention, no acceptance test,
no compaction) and imports neither the HIP binding nor the CPU oracle; both of
those consume the arrays made here.

The workloads stand in for the Spec-Bench / Vicuna-v1.3 runs of the paper's
experiment section (Sec. 4.1): head counts, head size and vocabulary follow the
model families named there, the tree shape follows the continuous verification
tree of Sec. 3.2 (a top-1 chain laid "vertically" first, then top-k siblings
added "horizontally").  No benchmark item, prompt or trained weight is involved.

All floating-point arrays are numpy; bf16 arrays are carried as ``uint16`` bit
patterns (round-to-nearest-even of the fp32 draw) so that every consumer sees
the same stored values.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence

import numpy as np

BASE_SEED = 250614158

# component ids for SeedSequence spawning (fixed, documented draw order)
_C_TREE, _C_Q, _C_KTREE, _C_VTREE, _C_KCACHE, _C_VCACHE = 1, 2, 3, 4, 5, 6
_C_LOGITS, _C_TOKENS, _C_PLANT, _C_DRAFT, _C_UNIF = 7, 8, 9, 10, 11
_C_RESAMPLE = 12


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    name: str
    index: int                 # 1..5 for the named configs, 0 for ad-hoc test shapes
    B: int
    Hq: int
    Hkv: int
    D: int
    dtype: str                 # "f32" | "bf16" | "f16"  (Q/K/V/cache/logits storage type)
    P: int                     # prefix length (cache_len[b] unless ragged)
    N: int                     # tree nodes including the root
    levels: int                # node levels including the root
    widths: Sequence[int]      # max children of a node at level l (None => complete binary)
    V: int
    mode: str                  # "greedy" | "stochastic"
    p_match: float = 0.7       # greedy: probability that a parent row gets a planted child
    qkv_std: float = 1.0
    temperature: float = 1.0
    complete_binary: bool = False
    ragged: bool = False       # draw cache_len[b] in [P/2, P] instead of P

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def S_cap(self) -> int:
        return self.P + self.N

    @property
    def es(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS = {
    1: VerifyConfig("tiny", 1, B=1, Hq=4, Hkv=4, D=64, dtype="f32", P=128, N=15, levels=4,
                    widths=(2, 2, 2), V=1000, mode="greedy", p_match=0.7, qkv_std=1.0,
                    complete_binary=True),
    2: VerifyConfig("7b", 2, B=1, Hq=32, Hkv=32, D=128, dtype="bf16", P=1024, N=60, levels=6,
                    widths=(4, 3, 2, 2, 1, 1), V=32000, mode="greedy", p_match=0.7,
                    qkv_std=1.0 / np.sqrt(128.0)),
    3: VerifyConfig("13b", 3, B=4, Hq=40, Hkv=40, D=128, dtype="bf16", P=4096, N=64, levels=7,
                    widths=(4, 3, 2, 2, 1, 1, 1, 1), V=32000, mode="stochastic"),
    4: VerifyConfig("gqa8b", 4, B=8, Hq=32, Hkv=8, D=128, dtype="bf16", P=8192, N=64, levels=8,
                    widths=(4, 3, 2, 2, 1, 1, 1, 1), V=128256, mode="greedy", p_match=0.6),
    5: VerifyConfig("70b-long", 5, B=16, Hq=64, Hkv=8, D=128, dtype="bf16", P=32768, N=128,
                    levels=10, widths=(8, 4, 3, 2, 2, 1, 1, 1, 1), V=128256, mode="stochastic"),
}


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def storage_type(dtype: str):
    """numpy element type of a config dtype: fp32 and fp16 natively, bf16 as uint16 bit patterns."""
    return {"f32": np.float32, "bf16": np.uint16, "f16": np.float16}[dtype]


def stored(x_f32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 draw -> storage array of the config dtype (round to nearest even)."""
    if dtype == "f32":
        return np.ascontiguousarray(x_f32, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x_f32, dtype=np.float32).astype(np.float16)
    return f32_to_bf16_bits(x_f32)


def as_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """storage array -> exact fp32 values."""
    if dtype == "f32":
        return x
    return x.astype(np.float32) if dtype == "f16" else bf16_bits_to_f32(x)


def _rng(seed: int, comp: int, b: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, comp, b]))


# --------------------------------------------------------------------------- trees
def complete_binary_parent(N: int) -> np.ndarray:
    p = np.empty(N, dtype=np.int32)
    p[0] = -1
    for i in range(1, N):
        p[i] = (i - 1) // 2
    return p


def random_tree_parent(N: int, levels: int, widths: Sequence[int], rng: np.random.Generator) -> np.ndarray:
    """Vertical-first, then horizontal growth (Sec. 3.2), relabelled in BFS order.

    Node 0 is the root.  A chain to the last level is laid first, then nodes are
    added one by one under a uniformly drawn eligible parent (not on the last
    level, fewer than widths[level] children).  Returned parent[] satisfies
    parent[0] = -1, parent[i] < i, and siblings are contiguous.
    """
    if N < levels:
        raise ValueError("N must be >= levels")
    par: List[int] = [-1]
    lev: List[int] = [0]
    nchild: List[int] = [0]
    for l in range(1, levels):                      # the top-1 chain
        par.append(len(par) - 1)
        lev.append(l)
        nchild.append(0)
        nchild[par[-1]] += 1
    while len(par) < N:
        elig = [i for i in range(len(par))
                if lev[i] < levels - 1 and nchild[i] < widths[min(lev[i], len(widths) - 1)]]
        if not elig:
            raise ValueError("tree capacity exhausted")
        u = elig[int(rng.integers(len(elig)))]
        par.append(u)
        lev.append(lev[u] + 1)
        nchild.append(0)
        nchild[u] += 1
    # BFS relabel: by level, then new index of the parent, then creation order
    new_of_old = {0: 0}
    order = [0]
    for l in range(1, levels):
        nodes = [i for i in range(len(par)) if lev[i] == l]
        nodes.sort(key=lambda i: (new_of_old[par[i]], i))
        for i in nodes:
            new_of_old[i] = len(order)
            order.append(i)
    out = np.empty(N, dtype=np.int32)
    for new, old in enumerate(order):
        out[new] = -1 if par[old] < 0 else new_of_old[par[old]]
    return out


def make_parent(cfg: VerifyConfig, seed: Optional[int] = None) -> np.ndarray:
    """parent[B][N] int32; trees are independent per sequence."""
    seed = cfg.seed() if seed is None else seed
    out = np.empty((cfg.B, cfg.N), dtype=np.int32)
    for b in range(cfg.B):
        if cfg.complete_binary:
            out[b] = complete_binary_parent(cfg.N)
        else:
            out[b] = random_tree_parent(cfg.N, cfg.levels, cfg.widths, _rng(seed, _C_TREE, b))
    return out


def children_lists(parent_row: np.ndarray) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in range(len(parent_row))]
    for i, p in enumerate(parent_row):
        if p >= 0:
            ch[int(p)].append(i)
    return ch


# --------------------------------------------------------------------------- attention inputs
@dataclasses.dataclass
class AttnInputs:
    q: np.ndarray          # [B][N][Hq][D]
    k_tree: np.ndarray     # [B][N][Hkv][D]
    v_tree: np.ndarray     # [B][N][Hkv][D]
    k_cache: np.ndarray    # [B][Hkv][S_cap][D]  rows >= cache_len[b] are zero
    v_cache: np.ndarray
    cache_len: np.ndarray  # [B] int32


def _normal(seed, comp, b, shape, std, dtype):
    x = _rng(seed, comp, b).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return stored(x, dtype)


def make_attn_inputs(cfg: VerifyConfig, seed: Optional[int] = None, threads: int = 8) -> AttnInputs:
    seed = cfg.seed() if seed is None else seed
    st = storage_type(cfg.dtype)
    B, N, Hq, Hkv, D, S = cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, cfg.S_cap
    if cfg.ragged:
        cache_len = _rng(seed, _C_KCACHE, 10_000).integers(cfg.P // 2, cfg.P + 1, size=B).astype(np.int32)
        cache_len[0] = cfg.P
    else:
        cache_len = np.full(B, cfg.P, dtype=np.int32)
    q = np.empty((B, N, Hq, D), dtype=st)
    kt = np.empty((B, N, Hkv, D), dtype=st)
    vt = np.empty((B, N, Hkv, D), dtype=st)
    kc = np.zeros((B, Hkv, S, D), dtype=st)
    vc = np.zeros((B, Hkv, S, D), dtype=st)

    def one(b):
        q[b] = _normal(seed, _C_Q, b, (N, Hq, D), cfg.qkv_std, cfg.dtype)
        kt[b] = _normal(seed, _C_KTREE, b, (N, Hkv, D), cfg.qkv_std, cfg.dtype)
        vt[b] = _normal(seed, _C_VTREE, b, (N, Hkv, D), cfg.qkv_std, cfg.dtype)
        L = int(cache_len[b])
        for h in range(Hkv):   # one head at a time keeps the fp32 temporaries small
            kc[b, h, :L] = _normal(seed, _C_KCACHE, b * Hkv + h, (L, D), cfg.qkv_std, cfg.dtype)
            vc[b, h, :L] = _normal(seed, _C_VCACHE, b * Hkv + h, (L, D), cfg.qkv_std, cfg.dtype)

    with ThreadPoolExecutor(max_workers=max(1, min(threads, B))) as ex:
        list(ex.map(one, range(B)))
    return AttnInputs(q, kt, vt, kc, vc, cache_len)


# --------------------------------------------------------------------------- acceptance inputs
@dataclasses.dataclass
class AcceptInputs:
    logits: np.ndarray     # [B][N][V] storage dtype; row i = target distribution after node i
    tokens: np.ndarray     # [B][N] int32
    p_draft: np.ndarray    # [B][N] float32 (stochastic; zeros in greedy)
    uniforms: np.ndarray   # [B][N] float32 in [0,1)
    draft_probs: Optional[np.ndarray] = None   # [B][N][V] float32: row u = draft distribution at node u (full_draft)
    u_resample: Optional[np.ndarray] = None    # [B] float32 in [0,1) for the correction token (full_draft)
    draft_logits: Optional[np.ndarray] = None  # [B][N][V] float32: the logits behind draft_probs (keep_draft_logits)


def _softmax64(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def draw_u_resample(seed: int, B: int, attempt: int = 0) -> np.ndarray:
    """[B] float32 uniforms for the correction token; attempt k re-draws them (test conditioning)."""
    return np.array([_rng(seed, _C_RESAMPLE, b + 100_000 * attempt).random(dtype=np.float32) for b in range(B)],
                    dtype=np.float32)


def make_accept_inputs(cfg: VerifyConfig, parent: np.ndarray, seed: Optional[int] = None,
                       threads: int = 8, full_draft: bool = False, keep_draft_logits: bool = False) -> AcceptInputs:
    """full_draft (stochastic mode only): also keep every internal node's whole draft
    distribution and draw the uniforms of the correction token; the other arrays are unchanged."""
    seed = cfg.seed() if seed is None else seed
    st = storage_type(cfg.dtype)
    B, N, V = cfg.B, cfg.N, cfg.V
    logits = np.empty((B, N, V), dtype=st)
    tokens = np.zeros((B, N), dtype=np.int32)
    p_draft = np.zeros((B, N), dtype=np.float32)
    uniforms = np.empty((B, N), dtype=np.float32)
    if full_draft and cfg.mode != "stochastic":
        raise ValueError("full_draft needs a stochastic config")
    draft_probs = np.zeros((B, N, V), dtype=np.float32) if full_draft else None
    if keep_draft_logits and cfg.mode != "stochastic":
        raise ValueError("keep_draft_logits needs a stochastic config")
    draft_logits = np.zeros((B, N, V), dtype=np.float32) if keep_draft_logits else None

    def one(b):
        logits[b] = _normal(seed, _C_LOGITS, b, (N, V), 2.0, cfg.dtype)
        rt = _rng(seed, _C_TOKENS, b)
        rp = _rng(seed, _C_PLANT, b)
        rd = _rng(seed, _C_DRAFT, b)
        uniforms[b] = _rng(seed, _C_UNIF, b).random(N, dtype=np.float32)
        tokens[b, 0] = int(rt.integers(V))
        ch = children_lists(parent[b])
        for u in range(N):
            k = len(ch[u])
            if k == 0:
                continue
            if cfg.mode == "greedy":
                toks = rt.choice(V, size=k, replace=False)
                tokens[b, ch[u]] = toks
                if rp.random() < cfg.p_match:
                    c = int(rp.integers(k))
                    row = as_f32(logits[b, u], cfg.dtype)
                    val = stored(np.array([row.max() + np.float32(1.0)], dtype=np.float32), cfg.dtype)
                    logits[b, u, int(toks[c])] = val[0]
                    chk = as_f32(logits[b, u], cfg.dtype)
                    assert int(np.argmax(chk)) == int(toks[c]) and (chk == chk.max()).sum() == 1
            else:
                row = as_f32(logits[b, u], cfg.dtype)
                dl = row + np.float32(0.5) * rd.standard_normal(V, dtype=np.float32)
                pd = _softmax64(dl)
                top = np.argsort(-pd, kind="stable")[:k]
                tokens[b, ch[u]] = top.astype(np.int32)
                p_draft[b, ch[u]] = pd[top].astype(np.float32)
                if full_draft:
                    draft_probs[b, u] = pd.astype(np.float32)
                if keep_draft_logits:
                    draft_logits[b, u] = dl

    with ThreadPoolExecutor(max_workers=max(1, min(threads, B))) as ex:
        list(ex.map(one, range(B)))
    return AcceptInputs(logits, tokens, p_draft, uniforms, draft_probs,
                        draw_u_resample(seed, B) if full_draft else None, draft_logits)


def levels_of(parent_row: np.ndarray) -> np.ndarray:
    """Level (root = 0) of every node; data-shape helper for sizing max_path."""
    lv = np.zeros(len(parent_row), dtype=np.int32)
    for i in range(1, len(parent_row)):
        lv[i] = lv[parent_row[i]] + 1
    return lv


def scaled(cfg: VerifyConfig, **kw) -> VerifyConfig:
    """A copy of a named config with some sizes overridden (parity-test shapes)."""
    return dataclasses.replace(cfg, **kw)
