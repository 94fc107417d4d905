"""GPU-vs-oracle parity of s4c_commit_path (all layers' K/V rows and the feature rows of the
accepted path in one call): cache bytes, cache_len, indices and feature rows bit-exact."""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.device import np_to_torch

pytestmark = pytest.mark.gpu


def bits(t):
    return t.view(torch.int16) if t.dtype in (torch.bfloat16, torch.float16) else t.view(torch.int32)


def random_paths(rng, parent, levels):
    """A root-to-node path per sequence (any node), -1 padded."""
    Bn, N = parent.shape
    path = np.full((Bn, levels), -1, dtype=np.int32)
    alen = np.zeros(Bn, dtype=np.int32)
    for b in range(Bn):
        node = int(rng.integers(0, N))
        chain = []
        while node >= 0:
            chain.append(node)
            node = int(parent[b, node])
        chain = chain[::-1]
        path[b, :len(chain)] = chain
        alen[b] = len(chain) - 1
    return path, alen


def stored_normal(rng, shape, dtype):
    x = rng.standard_normal(shape, dtype=np.float32)
    return x if dtype == "f32" else synth.f32_to_bf16_bits(x)


@pytest.mark.parametrize("dtype,Ly,Bn,Hkv,D,P,F", [("bf16", 4, 3, 2, 128, 300, 4096), ("f32", 2, 2, 4, 64, 40, 100),
                                                   ("bf16", 9, 5, 8, 128, 1000, 0), ("bf16", 1, 2, 1, 128, 0, 8)])
def test_commit_path_matches_the_oracle(dtype, Ly, Bn, Hkv, D, P, F):
    rng = np.random.default_rng(Ly * 100 + Bn)
    cfg = synth.scaled(synth.CONFIGS[3], B=Bn, index=0)
    N, levels = cfg.N, cfg.levels
    parent = synth.make_parent(cfg)
    path, alen = random_paths(rng, parent, levels)
    S_cap = P + levels
    cl = rng.integers(max(0, P - 5), P + 1, size=Bn).astype(np.int32)
    cl[-1] = S_cap - 1                                   # last sequence: overflows unless its path is the root alone
    kt = stored_normal(rng, (Ly, Bn, N, Hkv, D), dtype)
    vt = stored_normal(rng, (Ly, Bn, N, Hkv, D), dtype)
    kc = stored_normal(rng, (Ly, Bn, Hkv, S_cap, D), dtype)
    vc = stored_normal(rng, (Ly, Bn, Hkv, S_cap, D), dtype)
    feats = fout = None
    if F:
        feats = stored_normal(rng, (Bn, N, F), dtype)
        fout = stored_normal(rng, (Bn, levels, F), dtype)
    dev = lambda a: None if a is None else np_to_torch(a)
    d_kc, d_vc, d_fout = dev(kc), dev(vc), dev(fout)
    d_cl = torch.from_numpy(cl.copy()).cuda()
    d_dst = torch.full((Bn, levels), -9, dtype=torch.int32, device="cuda")
    d_st = torch.full((Bn,), -9, dtype=torch.int32, device="cuda")
    B.s4c_commit_path(dev(kt), dev(vt), d_kc, d_vc, d_cl, torch.from_numpy(path).cuda(), torch.from_numpy(alen).cuda(),
                      dev(feats), d_fout, d_dst, d_st)
    torch.cuda.synchronize()
    dst, st = O.commit_path(kt, vt, kc, vc, cl, path, alen, feats, fout)      # in place on kc, vc, cl, fout
    assert np.array_equal(d_st.cpu().numpy(), st) and np.array_equal(d_dst.cpu().numpy(), dst)
    assert np.array_equal(d_cl.cpu().numpy(), cl)
    assert torch.equal(bits(d_kc).cpu(), bits(np_to_torch(kc, "cpu")))
    assert torch.equal(bits(d_vc).cpu(), bits(np_to_torch(vc, "cpu")))
    if F:
        assert torch.equal(bits(d_fout).cpu(), bits(np_to_torch(fout, "cpu")))
    assert st[-1] == (2 if alen[-1] > 0 else 0)


def test_commit_path_equals_single_layer_calls_and_rejects_bad_arguments():
    cfg = synth.scaled(synth.CONFIGS[4], B=2, Hq=8, Hkv=2, P=64, index=0)
    par = synth.make_parent(cfg)
    at = synth.make_attn_inputs(cfg)
    rng = np.random.default_rng(5)
    path, alen = random_paths(rng, par, cfg.levels)
    Ly = 3
    t = lambda a: np_to_torch(np.stack([a] * Ly) if a.ndim == 4 else a)
    kt, vt = t(at.k_tree), t(at.v_tree)
    kt[1] += 1.0                                          # layers differ
    kc, vc = t(at.k_cache), t(at.v_cache)
    kc1, vc1 = kc.clone(), vc.clone()
    cl = torch.from_numpy(at.cache_len.copy()).cuda()
    cl1 = cl.clone()
    dp, da = torch.from_numpy(path).cuda(), torch.from_numpy(alen).cuda()
    B.s4c_commit_path(kt, vt, kc, vc, cl, dp, da)
    for l in range(Ly):
        c = cl1.clone()
        B.s4c_kv_compact(kt[l], vt[l], kc1[l], vc1[l], c, dp, da)
    torch.cuda.synchronize()
    assert torch.equal(bits(kc), bits(kc1)) and torch.equal(bits(vc), bits(vc1)) and torch.equal(cl, c)
    with pytest.raises(B.S4CError):                       # feature rows must be whole 16-byte units
        f = torch.zeros(2, cfg.N, 5, dtype=torch.float32, device="cuda")
        B.s4c_commit_path(kt, vt, kc, vc, cl, dp, da, f, torch.zeros(2, cfg.levels, 5, dtype=torch.float32, device="cuda"))


@pytest.mark.parametrize("dtype,Ly,Bn,Hkv,D,P,F,page", [("bf16", 4, 3, 2, 128, 300, 4096, 64), ("f32", 2, 2, 4, 64, 40, 96, 128),
                                                        ("f16", 3, 4, 8, 128, 1000, 0, 256)])
def test_commit_path_paged_matches_the_oracle(dtype, Ly, Bn, Hkv, D, P, F, page):
    """Paged pools [layers][num_pages][Hkv][page][D] behind one shuffled block table: pools, cache_len,
    destination rows, status and feature rows bit for bit; a bad page id and an overflow are flagged."""
    rng = np.random.default_rng(Ly * 100 + Bn + page)
    cfg = synth.scaled(synth.CONFIGS[3], B=Bn, index=0)
    N, levels = cfg.N, cfg.levels
    parent = synth.make_parent(cfg)
    path, alen = random_paths(rng, parent, levels)
    max_blocks = (P + levels + page - 1) // page
    S_log = max_blocks * page
    num_pages = Bn * max_blocks + 3
    bt = rng.permutation(num_pages)[:Bn * max_blocks].reshape(Bn, max_blocks).astype(np.int32)
    cl = rng.integers(max(0, P - 5), P + 1, size=Bn).astype(np.int32)
    cl[-1] = S_log - 1                                   # last sequence: overflows unless its path is the root alone
    if Bn > 2:
        bt[1, int(cl[1]) // page] = num_pages            # sequence 1: the page it would write to is not in the pool
    mk = (lambda shape: rng.standard_normal(shape, dtype=np.float32).astype(np.float16)) if dtype == "f16" else \
        (lambda shape: stored_normal(rng, shape, dtype))
    kt, vt = mk((Ly, Bn, N, Hkv, D)), mk((Ly, Bn, N, Hkv, D))
    kp, vp = mk((Ly, num_pages, Hkv, page, D)), mk((Ly, num_pages, Hkv, page, D))
    feats = fout = None
    if F:
        feats, fout = mk((Bn, N, F)), mk((Bn, levels, F))
    dev = lambda a: None if a is None else np_to_torch(a)
    d_kp, d_vp, d_fout = dev(kp), dev(vp), dev(fout)
    d_cl = torch.from_numpy(cl.copy()).cuda()
    d_dst = torch.full((Bn, levels), -9, dtype=torch.int32, device="cuda")
    d_st = torch.full((Bn,), -9, dtype=torch.int32, device="cuda")
    B.s4c_commit_path_paged(dev(kt), dev(vt), d_kp, d_vp, torch.from_numpy(bt).cuda(), d_cl, torch.from_numpy(path).cuda(),
                            torch.from_numpy(alen).cuda(), dev(feats), d_fout, d_dst, d_st)
    torch.cuda.synchronize()
    dst, st = O.commit_path_paged(kt, vt, kp, vp, bt, cl, path, alen, feats, fout)   # in place on kp, vp, cl, fout
    assert np.array_equal(d_st.cpu().numpy(), st) and np.array_equal(d_dst.cpu().numpy(), dst)
    assert np.array_equal(d_cl.cpu().numpy(), cl)
    assert torch.equal(bits(d_kp).cpu(), bits(np_to_torch(kp, "cpu")))
    assert torch.equal(bits(d_vp).cpu(), bits(np_to_torch(vp, "cpu")))
    if F:
        assert torch.equal(bits(d_fout).cpu(), bits(np_to_torch(fout, "cpu")))
    assert st[-1] == (2 if alen[-1] > 0 else 0)
    if Bn > 2:
        assert st[1] == 2
