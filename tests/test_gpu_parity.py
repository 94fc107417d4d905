"""GPU-vs-oracle parity through the C ABI (needs an MI355X: run with -m gpu).

Attention: element by element at sizes the oracle finishes in seconds (several tiles, ragged
tails, odd shapes); at the full config sizes, in the launch shape the benchmark times, every
output row of configs 2-4 and a sample of config 5 that hits every wavefront of the launch.  Tolerances: bf16 I/O with fp32 accumulation max abs <= 1e-2 and row-relative
<= 2e-2; fp32 <= 1e-5.  Acceptance and compaction: bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.verify import TreeVerifier
from paper_2506_14158_amd.device import np_to_torch as np_to_dev
from tests.util import accept_inputs_with_margin, attn_errors, to_device

pytestmark = pytest.mark.gpu

TOL = {"f32": (1e-5, 1e-5), "bf16": (1e-2, 2e-2), "f16": (2.5e-3, 2.5e-3)}
C = synth.CONFIGS


def verifier(cfg, d, max_cache_len=None):
    return TreeVerifier(cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, cfg.S_cap, cfg.V, d["q"].dtype if "q" in d else
                        {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[cfg.dtype], cfg.levels,
                        cfg.P if max_cache_len is None else max_cache_len)


# Outputs of magnitude >= 2 carry a storage rounding error of their own (half an ulp: 2^-9 |o| rounded
# up to the binade for bf16, 2^-12 for fp16) that a fixed absolute bar does not allow for; where a
# test produces such outputs on purpose the absolute bar is replaced by `floor + ulp_frac * |o|`.
ULP_BAR = {"f32": (1e-5, 0.0), "bf16": (5e-3, 2.0 ** -8), "f16": (1.25e-3, 2.0 ** -11)}


def check_attn_full(cfg, par=None, at=None, scale=0.0, ulp_aware=False, f32_slack=1.0):
    par = synth.make_parent(cfg) if par is None else par
    at = synth.make_attn_inputs(cfg) if at is None else at
    d = to_device(cfg, par, at)
    tv = verifier(cfg, d)
    tv.out.fill_(float("nan"))
    tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"], scale)
    torch.cuda.synchronize()
    ref, st = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par, scale)
    assert np.array_equal(tv.attn_status.cpu().numpy(), st)
    assert torch.isfinite(tv.out.float()).all()
    amax, rel = attn_errors(tv.out, ref)
    slack = f32_slack if cfg.dtype == "f32" else 1.0
    if ulp_aware:
        floor, frac = ULP_BAR[cfg.dtype]
        excess = float((np.abs(tv.out.float().cpu().numpy().astype(np.float64) - ref) - (slack * floor + frac * np.abs(ref))).max())
        assert excess <= 0 and rel <= slack * TOL[cfg.dtype][1], (cfg.name, amax, rel, excess)
    else:
        assert amax <= slack * TOL[cfg.dtype][0] and rel <= slack * TOL[cfg.dtype][1], (cfg.name, amax, rel)
    return tv, d, amax, rel


SMALL = [
    C[1],                                                                        # Tiny, as specified
    synth.scaled(C[1], name="tiny-noprefix", P=0, index=0),
    synth.scaled(C[1], name="tiny-b3-ragged", B=3, P=77, ragged=True, index=0),
    synth.scaled(C[1], name="f32-d128-gqa", Hq=6, Hkv=2, D=128, P=200, N=33, levels=6,
                 widths=(3, 2, 2, 2, 2), complete_binary=False, index=0),
    synth.scaled(C[2], name="7b-small", Hq=4, Hkv=4, P=333, index=0),            # ragged tail, N = 60
    synth.scaled(C[2], name="7b-splits", Hq=2, Hkv=2, P=2500, index=0),          # forces KV splits
    synth.scaled(C[3], name="13b-small", B=2, Hq=3, Hkv=3, P=1000, ragged=True, index=0),
    synth.scaled(C[4], name="gqa-small", B=2, Hq=8, Hkv=2, P=640, index=0),
    synth.scaled(C[5], name="70b-small", B=1, Hq=16, Hkv=2, P=520, index=0),     # N = 128, G = 8
    synth.scaled(C[4], name="gqa-n1", B=2, Hq=8, Hkv=2, P=130, N=1, levels=1, index=0),
    synth.scaled(C[4], name="gqa-d64", B=1, Hq=8, Hkv=4, D=64, P=257, N=37, levels=6, index=0),
    synth.scaled(C[4], name="gqa-p0", B=2, Hq=4, Hkv=1, P=0, N=50, levels=6, index=0),
    synth.scaled(C[4], name="gqa-p1", B=1, Hq=4, Hkv=1, P=1, N=17, levels=5, index=0),
    synth.scaled(C[2], name="7b-p0", Hq=2, Hkv=2, P=0, index=0),                 # few rows, tree only
    synth.scaled(C[3], name="13b-p70", B=2, Hq=2, Hkv=2, P=70, N=33, levels=6, index=0),
    synth.scaled(C[3], name="13b-p129", B=2, Hq=2, Hkv=1, P=129, N=32, levels=6, ragged=True, index=0),
    synth.scaled(C[5], name="70b-mid", B=1, Hq=8, Hkv=1, P=300, N=16, levels=5, index=0),   # M = 128: 4-wave kernel
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_tree_attn_elementwise(cfg):
    check_attn_full(cfg)


def _random_shapes():
    """Seeded sweep over shapes that land in each attention kernel (scalar; matrix-core with <= 64,
    <= 128 and > 128 query rows per KV head), with odd sizes, ragged lengths and forced KV splits."""
    rng = np.random.default_rng(20250614)
    shapes = []
    for k in range(20):
        dtype = "f32" if k % 5 == 4 else "bf16"
        D = 64 if (dtype == "f32" or k % 7 == 3) else 128
        G = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2, 3]))
        N = int(rng.integers(1, 129)) if k % 3 else int(rng.integers(1, 20))
        levels = 1 if N == 1 else int(min(N, rng.integers(2, 4) if N <= 9 else rng.integers(4, 9)))
        P = int(rng.choice([0, 1, 31, 63, 64, 65, 200, 777, 1500, 4100]))
        shapes.append(synth.scaled(C[4], name="rnd%d-%s-d%d-g%d-n%d-p%d" % (k, dtype, D, G, N, P), B=int(rng.integers(1, 4)),
                                   Hq=Hkv * G, Hkv=Hkv, D=D, dtype=dtype, P=P, N=N, levels=levels,
                                   widths=(8, 4, 3, 2, 2, 2, 2, 2), ragged=bool(k % 2) and P > 1, index=0))
    return shapes


@pytest.mark.parametrize("cfg", _random_shapes(), ids=lambda c: c.name)
def test_tree_attn_random_shapes(cfg):
    check_attn_full(cfg)


PEAKED = [
    synth.scaled(C[4], name="peaked-256rows", B=2, Hq=8, Hkv=2, P=3000, index=0),                   # 8 waves, 46 mask-free tiles
    synth.scaled(C[4], name="peaked-256rows-splits", B=1, Hq=4, Hkv=1, P=5000, ragged=False, index=0),
    synth.scaled(C[5], name="peaked-128rows", B=1, Hq=8, Hkv=1, P=1500, N=16, levels=5, index=0),   # 4 waves
    synth.scaled(C[3], name="peaked-64rows", B=2, Hq=3, Hkv=3, P=2000, ragged=True, index=0),       # key-group kernel
    synth.scaled(C[1], name="peaked-f32", B=2, P=300, index=0),                                      # scalar kernel
    synth.scaled(C[4], name="peaked-f16", B=2, Hq=8, Hkv=2, P=3000, dtype="f16", index=0),
]


@pytest.mark.parametrize("cfg", PEAKED, ids=lambda c: c.name)
def test_tree_attn_peaked_softmax(cfg):
    """Q and K scaled by 8 (exact in every storage type): scores of standard deviation ~64 instead of
    ~1, so the running maximum keeps jumping by far more than the slack the mask-free tiles allow
    before they rescale, and almost all weight sits on a few keys, so outputs are close to single V
    rows (magnitudes up to ~4: the absolute bar is the ulp-aware one).  For fp32 data the scores
    themselves are 64 times larger, and so is the fp32 rounding of the exponent's argument (~2^-24 x
    500 per score against the oracle's doubles): the fp32 bars are widened 16-fold here."""
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    times8 = lambda a: synth.stored(synth.as_f32(a, cfg.dtype) * np.float32(8.0), cfg.dtype)
    at = synth.AttnInputs(times8(at.q), times8(at.k_tree), at.v_tree, times8(at.k_cache), at.v_cache, at.cache_len)
    tv, d, amax, rel = check_attn_full(cfg, par=par, at=at, ulp_aware=True, f32_slack=16.0)
    print(cfg.name, "max abs %.2e rel %.2e" % (amax, rel))


def test_tree_attn_custom_scale_and_chain():
    cfg = synth.scaled(C[2], name="chain", Hq=2, Hkv=2, P=100, N=40, levels=40, index=0)
    par = np.arange(-1, cfg.N - 1, dtype=np.int32)[None]
    check_attn_full(cfg, par=par, scale=0.05)


def test_tree_attn_is_deterministic():
    cfg = synth.scaled(C[3], name="det", B=2, Hq=4, Hkv=4, P=3000, index=0)
    tv, d, _, _ = check_attn_full(cfg)
    first = tv.out.clone()
    for _ in range(3):
        tv.out.zero_()
        tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
        torch.cuda.synchronize()
        assert torch.equal(tv.out.view(torch.int16), first.view(torch.int16))


def test_tree_attn_flags_bad_sequences_and_zeroes_them():
    cfg = synth.scaled(C[4], name="bad", B=3, Hq=4, Hkv=2, P=300, N=20, levels=5, index=0)
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    par[1, 7] = 9                       # parent after child
    at.cache_len[2] = cfg.P + 5         # beyond max_cache_len
    d = to_device(cfg, par, at)
    tv = verifier(cfg, d)
    tv.out.fill_(float("nan"))
    tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
    torch.cuda.synchronize()
    assert tv.attn_status.cpu().tolist() == [0, B.S4C_SEQ_BAD_TREE, B.S4C_SEQ_BAD_LEN]
    assert (tv.out[1:] == 0).all()
    at.cache_len[2] = cfg.P
    ref, _ = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, synth.make_parent(cfg))
    amax, rel = attn_errors(tv.out[0], ref[0])
    assert amax <= 1e-2 and rel <= 2e-2


def test_tree_attn_beyond_two_billion_cache_elements():
    """Config 5's shape with 64 sequences: each of K and V holds 2.16e9 elements (4.3 GB), so every
    cache offset of the later sequences needs 64-bit arithmetic.  The cache is drawn on the device;
    the first and the last sequence are copied back and checked against the oracle on sampled rows."""
    cfg = synth.scaled(C[5], name="b64", B=64, index=0)
    Bn, N, Hq, Hkv, D, S = cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, cfg.S_cap
    assert Bn * Hkv * S * D > 2 ** 31
    g = torch.Generator(device="cuda").manual_seed(7)
    rn = lambda *s_: torch.randn(*s_, device="cuda", generator=g, dtype=torch.float32).bfloat16()
    kc = torch.empty(Bn, Hkv, S, D, dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    for b in range(Bn):                                   # per sequence: keeps the fp32 temporaries small
        kc[b] = rn(Hkv, S, D)
        vc[b] = rn(Hkv, S, D)
    q, kt, vt = rn(Bn, N, Hq, D), rn(Bn, N, Hkv, D), rn(Bn, N, Hkv, D)
    par = synth.make_parent(cfg)
    cl = torch.full((Bn,), cfg.P, dtype=torch.int32, device="cuda")
    tv = TreeVerifier(Bn, N, Hq, Hkv, D, S, 8, torch.bfloat16, cfg.levels, cfg.P)
    tv.tree_attn(q, kt, vt, kc, vc, cl, torch.from_numpy(par).cuda())
    torch.cuda.synchronize()
    assert tv.attn_status.cpu().tolist() == [0] * Bn
    pick = [0, Bn - 1]
    host = lambda t: np.ascontiguousarray(t[pick].view(torch.int16).cpu().numpy().view(np.uint16))
    rng = np.random.default_rng(3)
    n = 48
    tri = np.stack([rng.integers(0, 2, n), rng.integers(0, N, n), rng.integers(0, Hq, n)], 1).astype(np.int32)
    tri[0], tri[1] = (1, N - 1, Hq - 1), (0, 0, 0)
    ref = O.tree_attn_sampled(host(q), host(kt), host(vt), host(kc), host(vc), np.full(2, cfg.P, np.int32),
                              np.ascontiguousarray(par[pick]), tri)
    got = tv.out[pick][tri[:, 0], tri[:, 1], tri[:, 2]]
    amax, rel = attn_errors(got, ref)
    assert amax <= TOL["bf16"][0] and rel <= TOL["bf16"][1], (amax, rel)


def sample_triples(cfg, rng, n):
    t = np.stack([rng.integers(0, cfg.B, n), rng.integers(0, cfg.N, n), rng.integers(0, cfg.Hq, n)], 1).astype(np.int32)
    t[0] = (0, 0, 0)
    t[1] = (cfg.B - 1, cfg.N - 1, cfg.Hq - 1)
    return t


def stratified_triples(cfg, rng, per_cell, rows_per_wave=32):
    """(sequence, node, head) triples that hit every (sequence, KV head, query-row tile, wavefront) of
    the launch: the M = N*G query rows of a KV head are dealt out in blocks of rows_per_wave to the
    wavefronts of its workgroups; row r is node r // G, head kvh*G + r % G."""
    G = cfg.Hq // cfg.Hkv
    M = cfg.N * G
    out = []
    for b in range(cfg.B):
        for kvh in range(cfg.Hkv):
            for w0 in range(0, M, rows_per_wave):
                rows = rng.choice(np.arange(w0, min(M, w0 + rows_per_wave)), size=per_cell, replace=False)
                out += [(b, r // G, kvh * G + r % G) for r in rows]
    out += [(0, 0, 0), (cfg.B - 1, cfg.N - 1, cfg.Hq - 1)]
    return np.array(out, dtype=np.int32)


def _full_size_run(idx):
    cfg = C[idx]
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg, threads=16)
    d = to_device(cfg, par, at)
    tv = verifier(cfg, d)
    tv.out.fill_(float("nan"))
    tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
    torch.cuda.synchronize()
    out = tv.out.float().cpu().numpy()
    assert np.isfinite(out).all()
    assert tv.attn_status.cpu().tolist() == [0] * cfg.B
    return cfg, par, at, d, tv, out


def _root_rows_ignore_other_nodes(d, tv):
    # property that holds at any size: the root row of every head only sees prefix + itself, so it
    # must not change when every other tree node's K/V is scrambled
    kt2 = d["k_tree"].clone()
    kt2[:, 1:] = -kt2[:, 1:]
    root_before = tv.out[:, 0].clone()
    tv.tree_attn(d["q"], kt2, d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
    torch.cuda.synchronize()
    assert torch.equal(tv.out[:, 0].view(torch.int16), root_before.view(torch.int16))


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_tree_attn_full_size_every_row(idx):
    """Configs 2-4 at full size in the launch configuration the benchmark times: EVERY output row
    (1920 / 10240 / 16384 rows of 128) against the oracle."""
    cfg, par, at, d, tv, out = _full_size_run(idx)
    ref, st = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par)
    assert (st == 0).all()
    amax, rel = attn_errors(tv.out, ref)
    print("cfg%d all %d rows: max abs %.3e rel %.3e splits %d" % (idx, cfg.B * cfg.N * cfg.Hq, amax, rel, tv.num_splits))
    assert amax <= TOL["bf16"][0] and rel <= TOL["bf16"][1]
    _root_rows_ignore_other_nodes(d, tv)


def test_tree_attn_full_size_cfg5_stratified():
    """Config 5 at full size (131072 output rows; the oracle does ~700 of them per second): two rows
    from every (sequence, KV head, row tile, wavefront) of the 512-workgroup launch, 8194 rows."""
    cfg, par, at, d, tv, out = _full_size_run(5)
    bnh = stratified_triples(cfg, np.random.default_rng(5), per_cell=2)
    assert len(bnh) == cfg.B * cfg.Hkv * (cfg.N * cfg.G // 32) * 2 + 2
    ref = O.tree_attn_sampled(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par, bnh)
    got = out[bnh[:, 0], bnh[:, 1], bnh[:, 2]].astype(np.float64)
    amax = np.abs(got - ref).max()
    rel = (np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)).max()
    print("cfg5 stratified %d rows: max abs %.3e rel %.3e splits %d" % (len(bnh), amax, rel, tv.num_splits))
    assert amax <= 1e-2 and rel <= 2e-2
    _root_rows_ignore_other_nodes(d, tv)


def bf16_rne(x64):
    """float64 -> nearest bf16 value (ties to even), as float64."""
    return synth.as_f32(synth.f32_to_bf16_bits(x64.astype(np.float32)), "bf16").astype(np.float64)


def test_tree_attn_large_outputs_need_the_ulp_aware_bar():
    """Empty prefix, 122 nodes, 16 heads per KV head, N(0,1) values: a node attends to a handful of
    ancestors, so some outputs have magnitude 2..4, where the bf16 output's own half-ulp (2^-8 |o|
    rounded up to the binade: 0.0078) already uses up most of a fixed 1e-2 bar; this shape class
    measured max |g - o| = 0.0103.  The bar here is the ulp-aware one, and the claim that the excess
    is the output's storage rounding is checked directly: wherever |o| >= 1 the kernel's bf16 output
    is within one bf16 ulp of the correctly rounded oracle value."""
    cfg = synth.scaled(C[4], name="p0-n122-g16", B=4, Hq=48, Hkv=3, D=128, dtype="bf16", P=0, N=122, levels=7,
                       widths=(8, 4, 3, 2, 2, 2, 2, 2, 2), index=0)
    tv, d, amax, rel = check_attn_full(cfg, ulp_aware=True)
    at, par = synth.make_attn_inputs(cfg), synth.make_parent(cfg)
    ref, _ = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par)
    g = tv.out.float().cpu().numpy().astype(np.float64)
    big = np.abs(ref) >= 1.0
    assert big.sum() > 1000 and np.abs(ref).max() > 2.0          # the shape does produce such outputs
    ulp = 2.0 ** (np.floor(np.log2(np.abs(ref[big]))) - 7)
    assert (np.abs(g[big] - bf16_rne(ref[big])) <= ulp).all()
    print(cfg.name, "max abs %.3e rel %.3e, %d outputs with |o| >= 1, largest %.2f" % (amax, rel, big.sum(), np.abs(ref).max()))


# ------------------------------------------------------------------------------ acceptance
def run_accept(cfg, par, ac):
    d = to_device(cfg, par, None, ac)
    tv = verifier(cfg, d)
    mode = B.S4C_GREEDY if cfg.mode == "greedy" else B.S4C_STOCHASTIC
    for t in (tv.path, tv.accept_len, tv.accepted_tokens, tv.bonus_token):
        t.fill_(-7)
    tv.accept_path(d["logits"], d["parent"], d["tokens"], mode, d["p_draft"], d["uniforms"], cfg.temperature)
    torch.cuda.synchronize()
    return tv


def check_accept(cfg, par=None):
    par = synth.make_parent(cfg) if par is None else par
    ac, r = accept_inputs_with_margin(cfg, par, O)
    tv = run_accept(cfg, par, ac)
    assert np.array_equal(tv.accept_status.cpu().numpy(), r["status"])
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"])
    assert np.array_equal(tv.accepted_tokens.cpu().numpy(), r["accepted_tokens"])
    assert np.array_equal(tv.bonus_token.cpu().numpy(), r["bonus_token"])
    return r


ACCEPT_SMALL = [
    C[1],
    synth.scaled(C[1], name="tiny-v-odd", V=1003, B=3, index=0),                  # rows not 16-byte aligned
    synth.scaled(C[2], name="7b-v-odd", V=8191 * 3 + 5, index=0),
    synth.scaled(C[3], name="13b-small", B=2, V=9000, index=0),
    synth.scaled(C[3], name="13b-temp", B=2, V=9000, temperature=0.7, index=0),
    synth.scaled(C[5], name="70b-small", B=2, V=20000, index=0),
    synth.scaled(C[1], name="f32-stochastic", mode="stochastic", B=4, V=5000, N=31, levels=5, index=0),
    synth.scaled(C[2], name="7b-v-1m", B=2, V=1_000_003, N=9, levels=3, index=0),           # a million-token row, odd length
    synth.scaled(C[3], name="13b-v-1m", B=1, V=1_000_003, N=6, levels=3, index=0),
]


@pytest.mark.parametrize("cfg", ACCEPT_SMALL, ids=lambda c: c.name)
def test_accept_path_small(cfg):
    check_accept(cfg)


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_accept_path_full_size(idx):
    r = check_accept(C[idx])
    print("cfg%d accept_len" % idx, r["accept_len"].tolist())


def test_stochastic_acceptance_never_reads_leaf_rows():
    """A leaf's logits row verifies no node and the stochastic rule returns no bonus token: with every
    leaf row overwritten by NaN patterns the result must still be the oracle's on the clean rows."""
    cfg = synth.scaled(C[3], name="leaf-nan", B=3, V=9000, index=0)
    par = synth.make_parent(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    lg = ac.logits.copy()
    for b in range(cfg.B):
        has_child = np.zeros(cfg.N, dtype=bool)
        has_child[par[b, 1:]] = True
        lg[b, ~has_child] = 0x7FC0                       # bf16 quiet NaN
        assert (~has_child).sum() > 0
    ac2 = synth.AcceptInputs(lg, ac.tokens, ac.p_draft, ac.uniforms)
    tv = run_accept(cfg, par, ac2)
    assert np.array_equal(tv.accept_status.cpu().numpy(), r["status"])
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"])
    assert np.array_equal(tv.accepted_tokens.cpu().numpy(), r["accepted_tokens"])
    assert (tv.bonus_token.cpu().numpy() == -1).all()


def test_accept_repeated_calls_need_no_workspace_initialisation():
    """The acceptance workspace carries per-call tags instead of counters that would have to start at
    zero: the same answer must come out of many calls in a row, whatever the workspace held before each
    (zeros, the previous call's leftovers, random bytes), in both modes."""
    for cfg in (synth.scaled(C[1], name="rep-greedy", V=1003, B=3, index=0),
                synth.scaled(C[3], name="rep-stochastic", B=2, V=9000, index=0)):
        par = synth.make_parent(cfg)
        ac, r = accept_inputs_with_margin(cfg, par, O)
        d = to_device(cfg, par, None, ac)
        tv = verifier(cfg, d)
        mode = B.S4C_GREEDY if cfg.mode == "greedy" else B.S4C_STOCHASTIC
        g = torch.Generator(device="cuda").manual_seed(11)
        for it in range(12):
            if it % 3 == 0:
                tv.accept_ws.zero_()
            elif it % 3 == 1:
                tv.accept_ws.copy_(torch.randint(0, 256, tv.accept_ws.shape, device="cuda", generator=g, dtype=torch.int32).to(torch.uint8))
            for t in (tv.path, tv.accept_len, tv.accepted_tokens, tv.bonus_token, tv.accept_status):
                t.fill_(-7)
            tv.accept_path(d["logits"], d["parent"], d["tokens"], mode, d["p_draft"], d["uniforms"], cfg.temperature)
            torch.cuda.synchronize()
            assert np.array_equal(tv.accept_status.cpu().numpy(), r["status"]), (cfg.name, it)
            assert np.array_equal(tv.path.cpu().numpy(), r["path"]), (cfg.name, it)
            assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"]), (cfg.name, it)
            assert np.array_equal(tv.bonus_token.cpu().numpy(), r["bonus_token"]), (cfg.name, it)


def test_accept_collector_that_gives_up_flags_the_sequence(monkeypatch):
    """The bounded wait of the collecting workgroups, forced from the host: with a waiting time of zero a
    collector that does not find all of its sequence's statistics at its first look gives up.  The launch
    below has more scanning workgroups than fit on the GPU at once, and the collectors (which have no
    segment of their own in stochastic mode) are the last of the grid, so they start while the last
    scanning workgroups have only just begun 128 KB segments.  Every kernel must exit, the sequences
    must come back flagged and empty, and the next call with the default wait must give the oracle's
    answer on the same buffers."""
    cfg = synth.scaled(C[3], name="accept-timeout", B=2, V=1_000_003, index=0)
    par = synth.make_parent(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, None, ac)
    tv = verifier(cfg, d)
    call = lambda: tv.accept_path(d["logits"], d["parent"], d["tokens"], B.S4C_STOCHASTIC, d["p_draft"], d["uniforms"],
                                  cfg.temperature)
    monkeypatch.setenv("S4C_ACCEPT_WAIT_US", "0")
    for rep in range(2):
        for t in (tv.path, tv.accept_len, tv.accepted_tokens, tv.bonus_token, tv.accept_status):
            t.fill_(-7)
        call()
        torch.cuda.synchronize()
        assert tv.accept_status.cpu().tolist() == [B.S4C_SEQ_TIMEOUT] * cfg.B, rep
        assert tv.accept_len.cpu().tolist() == [0] * cfg.B and tv.bonus_token.cpu().tolist() == [-1] * cfg.B
        assert tv.path.cpu().tolist() == [[0] + [-1] * (cfg.levels - 1)] * cfg.B
        assert (tv.accepted_tokens.cpu().numpy() == -1).all()
    monkeypatch.delenv("S4C_ACCEPT_WAIT_US")
    call()
    torch.cuda.synchronize()
    assert np.array_equal(tv.accept_status.cpu().numpy(), r["status"])
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"])


def test_accept_argmax_ties_and_hand_example():
    """bf16 logits tie often; the lowest token id must win on the GPU exactly as in the oracle."""
    rng = np.random.default_rng(3)
    Bn, N, V = 2, 7, 40000
    lg = synth.f32_to_bf16_bits(np.round(rng.standard_normal((Bn, N, V)).astype(np.float32) * 2))   # integers: massive ties
    par = np.array([[-1, 0, 0, 1, 1, 2, 3]] * Bn, dtype=np.int32)
    g, _, _ = O.row_stats(lg.reshape(-1, V))
    g = g.reshape(Bn, N)
    tokens = np.zeros((Bn, N), dtype=np.int32)
    tokens[:, 1] = g[:, 0]; tokens[:, 2] = g[:, 0] + 1; tokens[:, 3] = g[:, 1] + 1; tokens[:, 4] = g[:, 1]
    tokens[:, 5] = g[:, 2]; tokens[:, 6] = g[:, 3]
    cfg = synth.scaled(C[2], name="ties", B=Bn, N=N, V=V, levels=4, index=0)
    ac = synth.AcceptInputs(lg, tokens, np.zeros((Bn, N), np.float32), np.zeros((Bn, N), np.float32))
    tv = run_accept(cfg, par, ac)
    r = O.accept_path(lg, par, tokens, "greedy", cfg.levels)
    assert tv.path.cpu().tolist() == [[0, 1, 4, -1]] * Bn == r["path"].tolist()
    assert np.array_equal(tv.bonus_token.cpu().numpy(), g[:, 4])


def test_accept_flags_bad_tree():
    cfg = synth.scaled(C[1], name="bad", B=3, index=0)
    par = synth.make_parent(cfg)
    par[1, 3] = 5
    par[2, 4] = -1                      # a second root
    ac = synth.make_accept_inputs(cfg, synth.make_parent(cfg))
    tv = run_accept(cfg, par, ac)
    r = O.accept_path(ac.logits, par, ac.tokens, "greedy", cfg.levels)
    assert tv.accept_status.cpu().tolist() == [0, 1, 1] == r["status"].tolist()
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"])
    assert np.array_equal(tv.bonus_token.cpu().numpy(), r["bonus_token"])


# ------------------------------------------------------------------------------ compaction + whole step
@pytest.mark.parametrize("cfg", [C[1], synth.scaled(C[4], name="gqa-small", B=3, P=300, V=5000, ragged=True, index=0),
                                 synth.scaled(C[5], name="70b-small", B=2, P=256, V=5000, index=0)],
                         ids=lambda c: c.name)
def test_whole_step_bit_exact_cache(cfg):
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, at, ac)
    tv = verifier(cfg, d)
    mode = B.S4C_GREEDY if cfg.mode == "greedy" else B.S4C_STOCHASTIC
    tv.step(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"],
            d["logits"], d["tokens"], mode, d["p_draft"], d["uniforms"], cfg.temperature)
    torch.cuda.synchronize()
    kc, vc, cl = at.k_cache.copy(), at.v_cache.copy(), at.cache_len.copy()
    dst, st = O.kv_compact(at.k_tree, at.v_tree, kc, vc, cl, r["path"], r["accept_len"])
    assert np.array_equal(tv.dst_index.cpu().numpy(), dst)
    assert np.array_equal(tv.compact_status.cpu().numpy(), st)
    assert np.array_equal(d["cache_len"].cpu().numpy(), cl)
    bits = lambda t: t.cpu().contiguous().view(torch.uint8).numpy()
    assert np.array_equal(bits(d["k_cache"]), kc.view(np.uint8))
    assert np.array_equal(bits(d["v_cache"]), vc.view(np.uint8))
    ref, _ = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par)
    amax, rel = attn_errors(tv.out, ref)
    assert amax <= TOL[cfg.dtype][0] and rel <= TOL[cfg.dtype][1]


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_kv_compact_full_size(idx):
    """The named configs at full size: the oracle's accepted paths appended by the GPU; destination
    rows, cache_len and every byte of both caches (appended rows and everything else) checked."""
    cfg = C[idx]
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg, threads=16)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, at)
    tv = verifier(cfg, d)
    tv.path.copy_(torch.from_numpy(r["path"]))
    tv.accept_len.copy_(torch.from_numpy(r["accept_len"]))
    tv.kv_compact(d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"])
    torch.cuda.synchronize()
    kc, vc, cl = at.k_cache, at.v_cache, at.cache_len.copy()          # the oracle works in place on the host copies
    dst, st = O.kv_compact(at.k_tree, at.v_tree, kc, vc, cl, r["path"], r["accept_len"])
    assert (st == 0).all() and tv.compact_status.cpu().tolist() == [0] * cfg.B
    assert np.array_equal(tv.dst_index.cpu().numpy(), dst)
    assert np.array_equal(d["cache_len"].cpu().numpy(), cl)
    assert int((cl - cfg.P).sum()) == int(r["accept_len"].sum()) + cfg.B
    for name, host in (("k_cache", kc), ("v_cache", vc)):
        assert torch.equal(d[name].view(torch.int16), np_to_dev(host).view(torch.int16)), name


def test_compact_rejects_overflow_and_bad_path():
    cfg = synth.scaled(C[1], name="ovf", B=3, index=0)
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    d = to_device(cfg, par, at)
    tv = verifier(cfg, d)
    path = np.array([[0, 1, 3, -1], [0, 2, 99, -1], [0, 1, 4, 9]], dtype=np.int32)
    alen = np.array([2, 2, 3], dtype=np.int32)
    cl = np.array([cfg.P, cfg.P, cfg.S_cap - 2], dtype=np.int32)      # seq 2: 4 rows do not fit
    tv.path.copy_(torch.from_numpy(path)); tv.accept_len.copy_(torch.from_numpy(alen))
    d["cache_len"].copy_(torch.from_numpy(cl))
    tv.kv_compact(d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"])
    torch.cuda.synchronize()
    kc, vc, cl2 = at.k_cache.copy(), at.v_cache.copy(), cl.copy()
    dst, st = O.kv_compact(at.k_tree, at.v_tree, kc, vc, cl2, path, alen)
    assert st.tolist() == [0, 2, 2] == tv.compact_status.cpu().tolist()
    assert np.array_equal(tv.dst_index.cpu().numpy(), dst)
    assert np.array_equal(d["cache_len"].cpu().numpy(), cl2)
    assert np.array_equal(d["k_cache"].cpu().numpy(), kc) and np.array_equal(d["v_cache"].cpu().numpy(), vc)


def test_step_replays_from_a_hip_graph():
    """The three calls allocate nothing, never synchronise and use no memset nodes, so a step can be
    captured once and replayed; every replay must reproduce the eager result."""
    cfg = synth.scaled(C[4], name="graph", B=2, Hq=8, Hkv=2, P=1500, V=9000, index=0)     # KV splits + merge
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, at, ac)
    tv = verifier(cfg, d)
    mode = B.S4C_GREEDY
    cl0 = d["cache_len"].clone()
    kc0, vc0 = d["k_cache"].clone(), d["v_cache"].clone()

    def step():
        tv.step(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"],
                d["logits"], d["tokens"], mode)
    step()                                  # eager reference
    torch.cuda.synchronize()
    ref = [t.clone() for t in (tv.out, tv.path, tv.accept_len, tv.bonus_token, d["cache_len"], d["k_cache"], d["v_cache"])]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    d["cache_len"].copy_(cl0); d["k_cache"].copy_(kc0); d["v_cache"].copy_(vc0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    for rep in range(3):
        d["cache_len"].copy_(cl0); d["k_cache"].copy_(kc0); d["v_cache"].copy_(vc0)       # eager work between replays
        tv.out.zero_(); tv.path.fill_(-9); tv.accept_len.fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (tv.out, tv.path, tv.accept_len, tv.bonus_token, d["cache_len"], d["k_cache"], d["v_cache"])
        for a_, b_ in zip(got, ref):
            assert torch.equal(a_.view(torch.uint8) if a_.dtype == torch.bfloat16 else a_,
                               b_.view(torch.uint8) if b_.dtype == torch.bfloat16 else b_), rep


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_consecutive_steps_share_one_growing_cache(dtype):
    """The continuous use of the step (Sec. 3.2: accepted tokens' features are kept for the following
    rounds): several rounds, each with a new tree, new Q and tree K/V and new logits, over ONE cache that
    the compaction of the round before has extended.  Every round's attention output, path and cache
    bytes must match the oracle run through the same rounds."""
    base = C[4] if dtype == "bf16" else C[1]
    cfg = synth.scaled(base, name="rounds-" + dtype, B=3, P=200, V=3000, ragged=True, mode="greedy", index=0,
                       **({"Hq": 8, "Hkv": 2} if dtype == "bf16" else {}))
    at = synth.make_attn_inputs(cfg)
    kc, vc, cl = at.k_cache.copy(), at.v_cache.copy(), at.cache_len.copy()       # the oracle's cache
    d_kc, d_vc = np_to_dev(kc), np_to_dev(vc)
    d_cl = torch.from_numpy(cl.copy()).cuda()
    tv = None
    grown = 0
    rounds = 4 if dtype == "bf16" else 3          # rows appended stay within S_cap = P + N
    for rnd in range(rounds):
        seed = cfg.seed() + 77 * (rnd + 1)
        par = synth.make_parent(cfg, seed=seed)
        a = synth.make_attn_inputs(cfg, seed=seed)                                # only q / k_tree / v_tree are used
        ac = synth.make_accept_inputs(cfg, par, seed=seed)
        d = to_device(cfg, par, None, ac)
        q, kt, vt = np_to_dev(a.q), np_to_dev(a.k_tree), np_to_dev(a.v_tree)
        if tv is None:
            tv = TreeVerifier(cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, cfg.S_cap, cfg.V, q.dtype, cfg.levels, cfg.S_cap)
        tv.step(q, kt, vt, d_kc, d_vc, d_cl, d["parent"], d["logits"], d["tokens"], B.S4C_GREEDY)
        torch.cuda.synchronize()
        ref, st = O.tree_attn(a.q, a.k_tree, a.v_tree, kc, vc, cl, par)           # on the cache BEFORE this round's append
        assert (st == 0).all() and tv.attn_status.cpu().tolist() == [0] * cfg.B
        amax, rel = attn_errors(tv.out, ref)
        assert amax <= TOL[dtype][0] and rel <= TOL[dtype][1], (rnd, amax, rel)
        r = O.accept_path(ac.logits, par, ac.tokens, "greedy", cfg.levels)
        assert np.array_equal(tv.path.cpu().numpy(), r["path"]), rnd
        dst, st2 = O.kv_compact(a.k_tree, a.v_tree, kc, vc, cl, r["path"], r["accept_len"])
        assert (st2 == 0).all() and tv.compact_status.cpu().tolist() == [0] * cfg.B
        assert np.array_equal(d_cl.cpu().numpy(), cl), rnd
        bits = lambda t: t.cpu().contiguous().view(torch.uint8).numpy()
        assert np.array_equal(bits(d_kc), kc.view(np.uint8)) and np.array_equal(bits(d_vc), vc.view(np.uint8)), rnd
        grown += int(r["accept_len"].sum()) + cfg.B
    assert int((cl - at.cache_len).sum()) == grown and grown >= rounds * cfg.B
