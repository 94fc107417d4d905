"""Pins of the oracle's fp16 path (CPU only).  fp16 is the storage precision of the paper's
experiments (Sec. 4.1, Evaluation and Environment); every oracle function decodes stored elements
through one routine, so the pins are (1) that routine against numpy's float16 -> float64 conversion
on all 65536 bit patterns, and (2) every entry point fed fp16 arrays against the same entry point
fed the same VALUES as fp32 arrays (fp16 values are exactly representable in fp32, so the double
results must be identical, not merely close)."""
import numpy as np

from oracle import s4c_oracle as O
from paper_2506_14158_amd import synth
from tests.test_oracle_attn import brute_force, rand_inputs, rand_parent


def test_decode_matches_numpy_on_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    got = O.decode(h)
    want = h.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))          # -0.0 keeps its sign
    # a few values written out by hand from the format definition
    hand = {0x3C00: 1.0, 0xC000: -2.0, 0x7BFF: 65504.0, 0x0001: 2.0 ** -24, 0x0400: 2.0 ** -14, 0x3555: 0.333251953125}
    for b, v in hand.items():
        assert O.decode(np.array([b], dtype=np.uint16).view(np.float16))[0] == v


def test_decode_of_the_other_types_is_exact_too():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(1000).astype(np.float32)
    assert np.array_equal(O.decode(x), x.astype(np.float64))
    b = synth.f32_to_bf16_bits(x)
    assert np.array_equal(O.decode(b), synth.bf16_bits_to_f32(b).astype(np.float64))


def test_attention_on_fp16_arrays_equals_attention_on_their_values():
    rng = np.random.default_rng(5)
    B, N, Hq, Hkv, D, P = 2, 9, 4, 2, 64, 21
    q, kt, vt, kc, vc = rand_inputs(rng, B, N, Hq, Hkv, D, P, dtype="f16")
    assert q.dtype == np.float16
    par = np.stack([rand_parent(rng, N) for _ in range(B)])
    cl = np.array([P, P - 4], dtype=np.int32)
    o16, s16 = O.tree_attn(q, kt, vt, kc, vc, cl, par)
    f = lambda a: a.astype(np.float32)
    o32, s32 = O.tree_attn(f(q), f(kt), f(vt), f(kc), f(vc), cl, par)
    assert np.array_equal(o16, o32) and np.array_equal(s16, s32)
    # and against the independent per-node brute force
    ref = brute_force(q, kt, vt, kc, vc, cl, par, "f16")
    np.testing.assert_allclose(o16, ref, rtol=1e-12, atol=1e-13)


def test_acceptance_tree_building_and_projection_on_fp16_arrays():
    rng = np.random.default_rng(6)
    cfg = synth.scaled(synth.CONFIGS[3], name="f16", B=2, N=12, V=700, levels=4, dtype="f16", index=0)
    par = synth.make_parent(cfg)
    ac = synth.make_accept_inputs(cfg, par, full_draft=True, keep_draft_logits=True)
    assert ac.logits.dtype == np.float16
    l32 = ac.logits.astype(np.float32)
    for mode in ("greedy", "stochastic"):
        a = O.accept_path(ac.logits, par, ac.tokens, mode, cfg.levels, ac.p_draft, ac.uniforms)
        b = O.accept_path(l32, par, ac.tokens, mode, cfg.levels, ac.p_draft, ac.uniforms)
        for k in a:
            assert np.array_equal(a[k], b[k]), (mode, k)
    a = O.accept_resample(ac.logits, ac.draft_probs, par, ac.tokens, ac.uniforms, ac.u_resample, cfg.levels)
    b = O.accept_resample(l32, ac.draft_probs, par, ac.tokens, ac.uniforms, ac.u_resample, cfg.levels)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    nchild = np.zeros_like(par)
    for bb in range(cfg.B):
        for i in range(1, cfg.N):
            nchild[bb, par[bb, i]] += 1
    dl16 = ac.draft_logits.astype(np.float16)
    a = O.build_tree(dl16, nchild, ac.tokens[:, 0], int(nchild.max()))
    b = O.build_tree(dl16.astype(np.float32), nchild, ac.tokens[:, 0], int(nchild.max()))
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    T, H, Hout = 5, 16, 8
    e, f_, W, bias = (rng.standard_normal(s).astype(np.float16) for s in ((T, H), (T, H), (Hout, 2 * H), (Hout,)))
    a = O.draft_linear(e, f_, W, bias)
    want = np.concatenate([e, f_], axis=1).astype(np.float64) @ W.astype(np.float64).T + bias.astype(np.float64)
    np.testing.assert_allclose(a, want, rtol=1e-13, atol=1e-13)


def test_compaction_moves_fp16_rows_bit_for_bit():
    rng = np.random.default_rng(8)
    B, N, Hkv, D, P = 2, 7, 2, 64, 10
    _, kt, vt, kc, vc = rand_inputs(rng, B, N, 2, Hkv, D, P, dtype="f16")
    cl = np.array([P, P - 3], dtype=np.int32)
    path = np.array([[0, 2, 5, -1], [0, 1, -1, -1]], dtype=np.int32)
    alen = np.array([2, 1], dtype=np.int32)
    k2, v2, c2 = kc.copy(), vc.copy(), cl.copy()
    dst, st = O.kv_compact(kt, vt, k2, v2, c2, path, alen)
    assert st.tolist() == [0, 0] and c2.tolist() == [P + 3, P - 3 + 2]
    for b in range(B):
        for j in range(alen[b] + 1):
            assert np.array_equal(k2[b, :, cl[b] + j].view(np.uint16), kt[b, path[b, j]].view(np.uint16))
            assert np.array_equal(v2[b, :, cl[b] + j].view(np.uint16), vt[b, path[b, j]].view(np.uint16))
