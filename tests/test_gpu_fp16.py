"""fp16 storage (IEEE binary16, the precision of the paper's experiments, Sec. 4.1) through every
entry point on the GPU, against the oracle.  Attention: max abs <= 2.5e-3 and row-relative <= 2.5e-3
(fp16 carries three more fraction bits than bf16, so rounding errors are 8x smaller; a quarter of
the bf16 bars); everything that decides integers is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.device import np_to_torch
from paper_2506_14158_amd.verify import TreeVerifier
from tests.util import accept_inputs_with_margin, attn_errors, to_device
from tests import test_gpu_build_tree as TB, test_gpu_parity as TP, test_gpu_resample as TR
from tests.test_gpu_paged import scatter_to_pool

pytestmark = pytest.mark.gpu
C = synth.CONFIGS
f16 = lambda c, **kw: synth.scaled(c, dtype="f16", index=0, **kw)

ATTN = [
    f16(C[1], name="tiny-f16"),                                                    # D = 64: scalar kernel
    f16(C[1], name="tiny-f16-ragged", B=3, P=77, ragged=True),
    f16(C[2], name="7b-f16", Hq=4, Hkv=4, P=333),                                  # <= 64 rows, ragged tail
    f16(C[2], name="7b-f16-splits", Hq=2, Hkv=2, P=2500),                          # KV splits + merge
    f16(C[3], name="13b-f16", B=2, Hq=3, Hkv=3, P=1000, ragged=True),
    f16(C[5], name="70b-f16-mid", B=1, Hq=8, Hkv=1, P=300, N=16, levels=5),        # 128 rows: 4-wave kernel
    f16(C[4], name="gqa-f16", B=2, Hq=8, Hkv=2, P=640),                            # 256 rows: 8-wave kernel
    f16(C[5], name="70b-f16", B=1, Hq=16, Hkv=2, P=520),                           # 1024 rows
    f16(C[4], name="gqa-f16-p0", B=2, Hq=4, Hkv=1, P=0, N=50, levels=6),           # tree only
    f16(C[4], name="gqa-f16-n1", B=2, Hq=8, Hkv=2, P=130, N=1, levels=1),
]


@pytest.mark.parametrize("cfg", ATTN, ids=lambda c: c.name)
def test_tree_attn_elementwise(cfg):
    tv, d, amax, rel = TP.check_attn_full(cfg)
    assert tv.out.dtype == torch.float16


def test_tree_attn_full_size_sampled_config5_shape():
    """Config 5's shape with fp16 data in the launch configuration the benchmark times."""
    cfg = synth.scaled(C[5], name="70b-long-f16", dtype="f16")
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg, threads=16)
    d = to_device(cfg, par, at)
    tv = TP.verifier(cfg, d)
    tv.out.fill_(float("nan"))
    tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"])
    torch.cuda.synchronize()
    out = tv.out.float().cpu().numpy()
    assert np.isfinite(out).all()
    bnh = TP.sample_triples(cfg, np.random.default_rng(50), 48)
    ref = O.tree_attn_sampled(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par, bnh)
    got = np.stack([out[b, i, h] for b, i, h in bnh]).astype(np.float64)
    amax = np.abs(got - ref).max()
    rel = (np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)).max()
    print("cfg5 fp16 sampled: max abs %.3e rel %.3e" % (amax, rel))
    assert amax <= 2.5e-3 and rel <= 2.5e-3


@pytest.mark.parametrize("cfg,page", [(f16(C[3], name="13b-f16", B=2, Hq=3, Hkv=3, P=1000, ragged=True), 64),
                                      (f16(C[4], name="gqa-f16", B=2, Hq=8, Hkv=2, P=640), 128),
                                      (f16(C[1], name="tiny-f16", B=2, P=200, ragged=True), 64)],
                         ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_paged_equals_contiguous(cfg, page):
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    d = to_device(cfg, par, at)
    kp, bt = scatter_to_pool(at.k_cache, page, np.random.default_rng(page))
    vp, _ = scatter_to_pool(at.v_cache, page, np.random.default_rng(page))
    S_log = bt.shape[1] * page
    tv = TreeVerifier(cfg.B, cfg.N, cfg.Hq, cfg.Hkv, cfg.D, S_log, cfg.V, d["q"].dtype, cfg.levels, cfg.P)
    out_p = torch.full_like(tv.out, float("nan"))
    B.s4c_tree_attn_paged(d["q"], d["k_tree"], d["v_tree"], np_to_torch(kp), np_to_torch(vp), np_to_torch(bt), d["cache_len"],
                          d["parent"], cfg.P, out_p, 0.0, None, tv.attn_ws)
    kc = torch.zeros(cfg.B, cfg.Hkv, S_log, cfg.D, dtype=d["q"].dtype, device="cuda")
    vc = torch.zeros_like(kc)
    kc[:, :, :cfg.S_cap] = d["k_cache"]
    vc[:, :, :cfg.S_cap] = d["v_cache"]
    tv.tree_attn(d["q"], d["k_tree"], d["v_tree"], kc, vc, d["cache_len"], d["parent"])
    torch.cuda.synchronize()
    assert torch.equal(out_p.view(torch.int16), tv.out.view(torch.int16))
    ref, _ = O.tree_attn(at.q, at.k_tree, at.v_tree, at.k_cache, at.v_cache, at.cache_len, par)
    amax, rel = attn_errors(out_p, ref)
    assert amax <= 2.5e-3 and rel <= 2.5e-3, (amax, rel)


ACCEPT = [
    f16(C[1], name="tiny-f16"),
    f16(C[1], name="tiny-f16-v-odd", V=1003, B=3),
    f16(C[2], name="7b-f16-v-odd", V=8191 * 3 + 5),
    f16(C[3], name="13b-f16", B=2, V=9000),
    f16(C[3], name="13b-f16-temp", B=2, V=9000, temperature=0.7),
    f16(C[5], name="70b-f16", B=2, V=20000),
    f16(C[4], name="gqa-f16-full-vocab", B=2),                                     # V = 128256
]


@pytest.mark.parametrize("cfg", ACCEPT, ids=lambda c: c.name)
def test_accept_path(cfg):
    TP.check_accept(cfg)


@pytest.mark.parametrize("cfg", [f16(C[3], name="13b-f16", B=3, V=9000), f16(C[3], name="13b-f16-v-odd", B=2, V=8191 * 3 + 5),
                                 f16(C[5], name="70b-f16", B=2, V=20000)], ids=lambda c: c.name)
def test_accept_resample(cfg):
    TR.check(cfg)


def test_build_tree_with_fp16_draft_logits():
    """fp16 rows tie often (as bf16 rows do): tokens, parents and levels bit-exact, lowest token id first."""
    cfg = f16(C[3], name="13b-f16", B=2, V=9000)
    par = synth.make_parent(cfg)
    rng = np.random.default_rng(4)
    dl = (2 * rng.standard_normal((cfg.B, cfg.N, cfg.V), dtype=np.float32)).astype(np.float16)
    nchild = TB.counts_of(par)
    kmax = int(nchild.max())
    root = np.arange(cfg.B, dtype=np.int32)
    g = TB.run(dl, nchild, root, kmax)
    r = O.build_tree(dl, nchild, root, kmax)
    TB.same(g, r)
    assert np.array_equal(g["parent"], par)


def test_whole_step_moves_fp16_rows_bit_for_bit():
    cfg = f16(C[4], name="gqa-f16-step", B=3, P=300, V=5000, ragged=True)
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, at, ac)
    tv = TP.verifier(cfg, d)
    tv.step(d["q"], d["k_tree"], d["v_tree"], d["k_cache"], d["v_cache"], d["cache_len"], d["parent"],
            d["logits"], d["tokens"], B.S4C_GREEDY, d["p_draft"], d["uniforms"], cfg.temperature)
    torch.cuda.synchronize()
    kc, vc, cl = at.k_cache.copy(), at.v_cache.copy(), at.cache_len.copy()
    dst, st = O.kv_compact(at.k_tree, at.v_tree, kc, vc, cl, r["path"], r["accept_len"])
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(d["cache_len"].cpu().numpy(), cl)
    bits = lambda t: t.cpu().contiguous().view(torch.uint8).numpy()
    assert np.array_equal(bits(d["k_cache"]), kc.view(np.uint8))
    assert np.array_equal(bits(d["v_cache"]), vc.view(np.uint8))


@pytest.mark.parametrize("T,H,Hout,bias", [(300, 64, 256, True), (777, 1024, 768, True), (2048, 512, 1024, False),
                                           (60, 4096, 4096, True), (128, 1056, 768, False), (15, 96, 256, True)])
def test_draft_linear(T, H, Hout, bias):
    """fp16 in/out, fp32 accumulate: |g - o| <= 2^-11 |o| + 3e-4 (half an ulp of the fp16 result plus the fp32 sum)."""
    rng = np.random.default_rng(T + H)
    h = lambda x: x.astype(np.float16)
    e, f_ = h(rng.standard_normal((T, H))), h(rng.standard_normal((T, H)))
    W = h(rng.standard_normal((Hout, 2 * H)) / np.sqrt(2 * H))
    b = h(rng.standard_normal(Hout)) if bias else None
    out = torch.full((T, Hout), float("nan"), dtype=torch.float16, device="cuda")
    B.s4c_draft_linear(np_to_torch(e), np_to_torch(f_), np_to_torch(W), out, None if b is None else np_to_torch(b),
                       B.alloc_workspace(B.s4c_draft_linear_workspace_size(e.shape[0], e.shape[1], W.shape[0])))
    torch.cuda.synchronize()
    g = out.float().cpu().numpy().astype(np.float64)
    o = O.draft_linear(e, f_, W, b)
    assert np.isfinite(g).all()
    err = np.abs(g - o)
    assert (err <= 2.0 ** -11 * np.abs(o) + 3e-4).all(), float((err - 2.0 ** -11 * np.abs(o)).max())
