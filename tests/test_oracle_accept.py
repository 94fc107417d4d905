"""Pins of the oracle's acceptance / longest-path step (Sec. 3.2) and of compaction (CPU only)."""
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import s4c_oracle as O
from paper_2506_14158_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def logits_with_argmax(rng, g, V):
    lg = rng.standard_normal((len(g), V)).astype(np.float32)
    for r, t in enumerate(g):
        lg[r, t] = lg[r].max() + 1.0
    return lg


def read_examples():
    ex = []
    for line in open(os.path.join(GOLD, "accept_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        ints = lambda s: [int(x) for x in s.split()]
        ex.append((f[0], ints(f[1]), ints(f[2]), ints(f[3]), ints(f[4]), ints(f[5]), int(f[6])))
    return ex


@pytest.mark.parametrize("ex", read_examples(), ids=lambda e: e[0])
def test_greedy_hand_examples(ex):
    name, parent, tokens, g, path, atoks, bonus = ex
    rng = np.random.default_rng(1)
    lg = logits_with_argmax(rng, g, 128)[None]
    r = O.accept_path(lg, np.array([parent]), np.array([tokens]), "greedy", max_path=6)
    L = len(path) - 1
    assert r["accept_len"][0] == L
    assert list(r["path"][0]) == path + [-1] * (6 - len(path))
    assert list(r["accepted_tokens"][0]) == atoks + [-1] * (6 - len(atoks))
    assert r["bonus_token"][0] == bonus
    assert r["status"][0] == 0


def rows_from_probs(probs):
    """logits rows whose softmax is exactly the given distribution (log-probabilities)."""
    return np.log(np.asarray(probs, dtype=np.float64)).astype(np.float32)


def test_stochastic_chain_example():
    """Chain 0-1-2-3, V = 4.  Target probabilities of the drafted tokens (0.5, 0.2, 0.4), draft
    probabilities (0.4, 0.5, 0.4).  u = (0.9, 0.3, 0.999): 0.36 < 0.5, 0.15 < 0.2, 0.3996 < 0.4
    -> all three accepted.  With u_2 = 0.45: 0.225 >= 0.2 -> node 2 fails -> length 1."""
    parent = np.array([[-1, 0, 1, 2]])
    tokens = np.array([[0, 1, 2, 3]])
    rows = rows_from_probs([[0.1, 0.5, 0.3, 0.1],     # row of node 0: token 1 has 0.5
                            [0.3, 0.3, 0.2, 0.2],     # row of node 1: token 2 has 0.2
                            [0.2, 0.2, 0.2, 0.4],     # row of node 2: token 3 has 0.4
                            [0.25, 0.25, 0.25, 0.25]])[None]
    pd = np.array([[0.0, 0.4, 0.5, 0.4]], dtype=np.float32)
    u = np.array([[0.0, 0.9, 0.3, 0.999]], dtype=np.float32)
    r = O.accept_path(rows, parent, tokens, "stochastic", 4, pd, u)
    assert r["accept_len"][0] == 3 and list(r["path"][0]) == [0, 1, 2, 3]
    assert list(r["accepted_tokens"][0]) == [1, 2, 3, -1] and r["bonus_token"][0] == -1
    # smallest margin is node 3: |0.3996 - 0.4| / 0.4 = 1e-3
    assert abs(r["margin"][0] - 1e-3) < 1e-5
    u2 = u.copy()
    u2[0, 2] = 0.45
    r = O.accept_path(rows, parent, tokens, "stochastic", 4, pd, u2)
    assert r["accept_len"][0] == 1 and list(r["path"][0]) == [0, 1, -1, -1]


def test_stochastic_longest_not_first():
    """Two children pass at level 1; only the second has a passing child: deepest path wins."""
    parent = np.array([[-1, 0, 0, 1, 2]])
    tokens = np.array([[0, 1, 2, 3, 3]])
    rows = rows_from_probs([[0.1, 0.4, 0.4, 0.1], [0.7, 0.1, 0.1, 0.1], [0.1, 0.1, 0.1, 0.7],
                            [0.25] * 4, [0.25] * 4])[None]
    pd = np.array([[0, 0.4, 0.4, 0.5, 0.5]], dtype=np.float32)
    u = np.array([[0, 0.5, 0.5, 0.5, 0.5]], dtype=np.float32)   # n3: .25 >= .1 fails ; n4: .25 < .7 passes
    r = O.accept_path(rows, parent, tokens, "stochastic", 3, pd, u)
    assert list(r["path"][0]) == [0, 2, 4] and r["accept_len"][0] == 2


def test_strict_inequality_and_temperature():
    """u*pd == pt exactly must reject (strict '<').  Two-token row with equal logits gives
    pt = 0.5 exactly; pd = 1, u = 0.5 -> reject, u just below -> accept.  Temperature:
    logits (ln 4, 0) at T = 2 give pt = 2/3 for token 0."""
    parent = np.array([[-1, 0]])
    tokens = np.array([[0, 0]])
    rows = np.zeros((1, 2, 2), dtype=np.float32)
    pd = np.array([[0, 1.0]], dtype=np.float32)
    r = O.accept_path(rows, parent, tokens, "stochastic", 2, pd, np.array([[0, 0.5]], np.float32))
    assert r["accept_len"][0] == 0 and r["margin"][0] == 0.0
    r = O.accept_path(rows, parent, tokens, "stochastic", 2, pd, np.array([[0, np.nextafter(np.float32(0.5), np.float32(0))]], np.float32))
    assert r["accept_len"][0] == 1
    rows[0, 0] = [np.log(4.0), 0.0]
    for u, want in ((0.66, 1), (0.67, 0)):
        r = O.accept_path(rows, parent, tokens, "stochastic", 2, pd, np.array([[0, u]], np.float32), temperature=2.0)
        assert r["accept_len"][0] == want


def test_chain_equals_sequential_speculative_sampling():
    """On a chain the rule is the sequential one of Sec. 2: walk the drafts in order, keep token
    i while u_i < min(1, target/draft), stop at the first failure.  Reference uses scipy."""
    rng = np.random.default_rng(5)
    for trial in range(40):
        N, V = 9, 50
        T = [1.0, 0.7, 1.5][trial % 3]
        parent = np.arange(-1, N - 1, dtype=np.int32)[None]
        lg = (2 * rng.standard_normal((1, N, V))).astype(np.float32)
        tokens = rng.integers(0, V, size=(1, N)).astype(np.int32)
        pd = rng.uniform(0.01, 0.3, size=(1, N)).astype(np.float32)
        u = rng.random((1, N), dtype=np.float32)
        want = 0
        for i in range(1, N):
            pt = softmax(lg[0, i - 1].astype(np.float64) / T)[tokens[0, i]]
            if float(u[0, i]) < min(1.0, pt / float(pd[0, i])):
                want += 1
            else:
                break
        r = O.accept_path(lg, parent, tokens, "stochastic", N, pd, u, temperature=T)
        assert r["accept_len"][0] == want
        assert list(r["path"][0][:want + 1]) == list(range(want + 1))


def test_u_zero_accepts_deepest_lowest_index_leaf_and_u_one_rejects():
    rng = np.random.default_rng(6)
    parent = np.array([[-1, 0, 0, 1, 1, 2, 2, 3, 6]])       # depth 3 nodes: 7 (under 3) and 8 (under 6)
    N, V = 9, 30
    lg = rng.standard_normal((1, N, V)).astype(np.float32)
    tokens = rng.integers(0, V, (1, N)).astype(np.int32)
    pd = np.full((1, N), 0.2, np.float32)
    r = O.accept_path(lg, parent, tokens, "stochastic", 4, pd, np.zeros((1, N), np.float32))
    assert list(r["path"][0]) == [0, 1, 3, 7] and r["accept_len"][0] == 3
    # draft prob 1 and u -> 1 : u*pd ~ 1 > any pt -> nothing accepted
    r = O.accept_path(lg, parent, tokens, "stochastic", 4, np.ones((1, N), np.float32),
                      np.full((1, N), np.nextafter(np.float32(1), np.float32(0)), np.float32))
    assert r["accept_len"][0] == 0 and list(r["path"][0]) == [0, -1, -1, -1]


def test_row_stats_vs_numpy_scipy_and_tie_break():
    rng = np.random.default_rng(7)
    lg = synth.stored((2 * rng.standard_normal((12, 777))).astype(np.float32), "bf16")
    f = synth.bf16_bits_to_f32(lg).astype(np.float64)
    # bf16 rows have many exact ties near the top; force one at the maximum too
    lg[3, 700] = lg[3, 5] = synth.f32_to_bf16_bits(np.array([f[3].max() + 1], np.float32))[0]
    f = synth.bf16_bits_to_f32(lg).astype(np.float64)
    g, m, S = O.row_stats(lg, temperature=1.3)
    np.testing.assert_array_equal(g, np.argmax(f, axis=1))      # numpy argmax = first occurrence
    assert g[3] == 5
    np.testing.assert_array_equal(m, f.max(axis=1))
    np.testing.assert_allclose(np.log(S) + m / 1.3, logsumexp(f / 1.3, axis=1), rtol=1e-12)


def test_greedy_ties_pick_lowest_token_id():
    lg = np.zeros((1, 2, 8), dtype=np.float32)
    lg[0, 0, [2, 6]] = 5.0                                  # tie: argmax is token 2
    parent = np.array([[-1, 0]])
    assert O.accept_path(lg, parent, np.array([[0, 2]]), "greedy", 2)["accept_len"][0] == 1
    assert O.accept_path(lg, parent, np.array([[0, 6]]), "greedy", 2)["accept_len"][0] == 0


def test_malformed_tree_and_short_max_path_flagged():
    lg = np.zeros((1, 3, 4), dtype=np.float32)
    r = O.accept_path(lg, np.array([[-1, 0, 2]]), np.array([[0, 0, 0]]), "greedy", 3)
    assert r["status"][0] == 1 and r["accept_len"][0] == 0 and list(r["path"][0]) == [0, -1, -1]
    r = O.accept_path(lg, np.array([[-1, -1, 0]]), np.array([[0, 0, 0]]), "greedy", 3)   # second root
    assert r["status"][0] == 1
    r = O.accept_path(lg, np.array([[-1, 0, 1]]), np.array([[0, 0, 0]]), "greedy", 2)    # depth 2 needs 3 slots
    assert r["status"][0] == 1


# ----------------------------------------------------------------------------- compaction
def test_compaction_equals_appending_one_by_one_then_decoding():
    """After compaction the cache must be what appending the accepted tokens one at a time
    would have produced, and ordinary attention of a new query over it must equal tree
    attention of a child of the last accepted node."""
    rng = np.random.default_rng(8)
    B, N, Hq, Hkv, D, P = 2, 8, 4, 2, 8, 5
    S_cap = P + N
    mk = lambda *s: rng.standard_normal(s).astype(np.float32)
    q, kt, vt = mk(B, N, Hq, D), mk(B, N, Hkv, D), mk(B, N, Hkv, D)
    kc, vc = mk(B, Hkv, S_cap, D), mk(B, Hkv, S_cap, D)
    parent = np.array([[-1, 0, 0, 1, 1, 2, 4, 6]] * B, dtype=np.int32)
    cl = np.array([P, P - 2], dtype=np.int32)
    path = np.array([[0, 1, 4, 6], [0, 2, -1, -1]], dtype=np.int32)
    alen = np.array([3, 1], dtype=np.int32)
    kc2, vc2, cl2 = kc.copy(), vc.copy(), cl.copy()
    dst, st = O.kv_compact(kt, vt, kc2, vc2, cl2, path, alen)
    assert (st == 0).all()
    # reference: python appends
    for b in range(B):
        kref, vref, n = kc[b].copy(), vc[b].copy(), int(cl[b])
        for k in range(alen[b] + 1):
            kref[:, n] = kt[b, path[b, k]]
            vref[:, n] = vt[b, path[b, k]]
            assert dst[b, k] == n
            n += 1
        assert cl2[b] == n and (dst[b, alen[b] + 1:] == -1).all()
        np.testing.assert_array_equal(kc2[b], kref)
        np.testing.assert_array_equal(vc2[b], vref)
    # decode equivalence for sequence 0: node 7 is a child of node 6 (the last accepted node)
    full, _ = O.tree_attn(q, kt, vt, kc, vc, cl, parent)
    q1, k1, v1 = (np.ascontiguousarray(x[:, 7:8]) for x in (q, kt, vt))
    dec, _ = O.tree_attn(q1, k1, v1, kc2, vc2, cl2, np.full((B, 1), -1, np.int32))
    np.testing.assert_allclose(dec[0, 0], full[0, 7], rtol=1e-12, atol=1e-14)


def test_compaction_overflow_is_rejected_untouched():
    rng = np.random.default_rng(9)
    kt = rng.standard_normal((1, 4, 1, 4)).astype(np.float32)
    kc = rng.standard_normal((1, 1, 6, 4)).astype(np.float32)
    kc0 = kc.copy()
    vc = kc.copy()
    cl = np.array([5], np.int32)
    dst, st = O.kv_compact(kt, kt, kc, vc, cl, np.array([[0, 1, 3]], np.int32), np.array([2], np.int32))
    assert st[0] == 2 and cl[0] == 5 and (dst == -1).all()
    np.testing.assert_array_equal(kc, kc0)


# ----------------------------------------------------------------------------- generators
def test_generated_workloads_have_the_stated_structure():
    for idx in (1, 2):
        cfg = synth.CONFIGS[idx]
        par = synth.make_parent(cfg)
        assert par.shape == (cfg.B, cfg.N) and (par[:, 0] == -1).all()
        for b in range(cfg.B):
            assert all(0 <= par[b, i] < i for i in range(1, cfg.N))
            lv = synth.levels_of(par[b])
            assert lv.max() == cfg.levels - 1 and (np.diff(lv) >= 0).all()      # BFS order
            ch = synth.children_lists(par[b])
            for u, c in enumerate(ch):
                assert len(c) <= cfg.widths[min(lv[u], len(cfg.widths) - 1)]
                assert c == list(range(c[0], c[0] + len(c))) if c else True     # siblings contiguous
        acc = synth.make_accept_inputs(cfg, par)
        r = O.accept_path(acc.logits, par, acc.tokens, "greedy", cfg.levels)
        assert 0 <= r["accept_len"][0] < cfg.levels
    small = synth.scaled(synth.CONFIGS[3], B=2, V=2000, N=24, levels=5)
    par = synth.make_parent(small)
    acc = synth.make_accept_inputs(small, par)
    assert (acc.p_draft[:, 1:] > 0).all() and (acc.uniforms >= 0).all() and (acc.uniforms < 1).all()
    # siblings are the draft's top-k in decreasing probability
    ch = synth.children_lists(par[0])
    for c in ch:
        if len(c) > 1:
            assert (np.diff(acc.p_draft[0, c]) <= 0).all() and len(set(acc.tokens[0, c])) == len(c)
    a2 = synth.make_accept_inputs(small, par)
    np.testing.assert_array_equal(acc.logits, a2.logits)                           # seeded => reproducible
    r = O.accept_path(acc.logits, par, acc.tokens, "stochastic", small.levels, acc.p_draft, acc.uniforms)
    assert (r["status"] == 0).all()


# ------------------------------------------------------------------------------ multi-layer commit
def test_commit_path_equals_per_layer_compaction_and_feature_gather():
    """All layers in one call == the single-layer routine applied layer by layer from the same
    cache_len, and the feature rows == a plain numpy gather of the path's nodes."""
    rng = np.random.default_rng(17)
    Ly, B, N, Hkv, D, P, mp, F = 3, 4, 9, 2, 8, 5, 5, 6
    S_cap = P + 4                                                    # sequence 3 overflows
    kt = rng.standard_normal((Ly, B, N, Hkv, D)).astype(np.float32)
    vt = rng.standard_normal((Ly, B, N, Hkv, D)).astype(np.float32)
    kc = rng.standard_normal((Ly, B, Hkv, S_cap, D)).astype(np.float32)
    vc = rng.standard_normal((Ly, B, Hkv, S_cap, D)).astype(np.float32)
    cl = np.array([P, P - 2, 0, P], dtype=np.int32)
    path = np.array([[0, 2, 5, -1, -1], [0, -1, -1, -1, -1], [0, 1, 3, 7, -1], [0, 1, 4, 6, 8]], dtype=np.int32)
    alen = np.array([2, 0, 3, 4], dtype=np.int32)
    feats = rng.standard_normal((B, N, F)).astype(np.float32)
    fout = np.full((B, mp, F), -5.0, dtype=np.float32)
    kc1, vc1, cl1, fout1 = kc.copy(), vc.copy(), cl.copy(), fout.copy()
    dst, st = O.commit_path(kt, vt, kc1, vc1, cl1, path, alen, feats, fout1)
    assert st.tolist() == [0, 0, 0, 2]
    for l in range(Ly):
        kcl, vcl, cll = kc[l].copy(), vc[l].copy(), cl.copy()
        d2, s2 = O.kv_compact(kt[l], vt[l], kcl, vcl, cll, path, alen)
        assert np.array_equal(kcl, kc1[l]) and np.array_equal(vcl, vc1[l])
        assert np.array_equal(cll, cl1) and np.array_equal(d2, dst) and np.array_equal(s2, st)
    want = fout.copy()
    for b in range(3):
        want[b, :alen[b] + 1] = feats[b, path[b, :alen[b] + 1]]
    assert np.array_equal(fout1, want)                               # flagged sequence 3 and padding rows untouched
    # no features: same caches
    kc2, vc2, cl2 = kc.copy(), vc.copy(), cl.copy()
    O.commit_path(kt, vt, kc2, vc2, cl2, path, alen)
    assert np.array_equal(kc2, kc1) and np.array_equal(cl2, cl1)


# ------------------------------------------------------------------------------ paged cache
def _paged_copy_of(cache, cache_len, page_size, rng, spare=3):
    """Scatter a contiguous cache [B][Hkv][S][D] into a pool through a random block table."""
    B, Hkv, S, D = cache.shape
    max_blocks = (S + page_size - 1) // page_size
    num_pages = B * max_blocks + spare
    perm = rng.permutation(num_pages)
    bt = perm[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
    pool = rng.standard_normal((num_pages, Hkv, page_size, D)).astype(cache.dtype)     # junk everywhere else
    for b in range(B):
        for j in range(S):
            pool[bt[b, j // page_size], :, j % page_size] = cache[b, :, j]
    return pool, bt


def test_paged_gather_and_paged_compaction_match_the_contiguous_layout():
    rng = np.random.default_rng(23)
    B, N, Hkv, D, S, ps = 3, 9, 2, 8, 40, 16
    kc = rng.standard_normal((B, Hkv, S, D)).astype(np.float32)
    vc = rng.standard_normal((B, Hkv, S, D)).astype(np.float32)
    cl = np.array([20, 33, 0], dtype=np.int32)
    for b in range(B):
        kc[b, :, cl[b]:] = 0
        vc[b, :, cl[b]:] = 0
    kp, bt = _paged_copy_of(kc, cl, ps, rng)
    vp = np.empty_like(kp)
    for b in range(B):
        for j in range(S):
            vp[bt[b, j // ps], :, j % ps] = vc[b, :, j]
    # gather inverts the scatter on the valid rows, zero elsewhere
    g, st = O.paged_gather(kp, bt, cl, S)
    assert st.tolist() == [0, 0, 0] and np.array_equal(g, kc)
    # compaction: paged == contiguous, seen through the block table
    kt = rng.standard_normal((B, N, Hkv, D)).astype(np.float32)
    vt = rng.standard_normal((B, N, Hkv, D)).astype(np.float32)
    path = np.array([[0, 2, 5, -1], [0, -1, -1, -1], [0, 1, 3, 7]], dtype=np.int32)
    alen = np.array([2, 0, 3], dtype=np.int32)
    kc2, vc2, cl2 = kc.copy(), vc.copy(), cl.copy()
    d1, s1 = O.kv_compact(kt, vt, kc2, vc2, cl2, path, alen)
    clp = cl.copy()
    d2, s2 = O.kv_compact_paged(kt, vt, kp, vp, bt, clp, path, alen)
    assert np.array_equal(d1, d2) and np.array_equal(s1, s2) and np.array_equal(cl2, clp)
    gk, _ = O.paged_gather(kp, bt, clp, S)
    gv, _ = O.paged_gather(vp, bt, clp, S)
    assert np.array_equal(gk, kc2) and np.array_equal(gv, vc2)
    # a page id outside the pool flags the sequence and leaves it alone
    bt_bad = bt.copy()
    bt_bad[1, 2] = kp.shape[0]
    g, st = O.paged_gather(kp, bt_bad, clp, S)
    assert st.tolist() == [0, 2, 0] and (g[1] == 0).all() and np.array_equal(g[0], kc2[0])
    kp3, clq = kp.copy(), clp.copy()
    d3, s3 = O.kv_compact_paged(kt, vt, kp3, vp.copy(), bt_bad, clq, path, alen)
    assert s3.tolist() == [0, 2, 0] and clq[1] == clp[1]


def test_paged_multi_layer_commit_matches_the_contiguous_one_and_plain_numpy():
    """oracle_commit_path_paged against (1) oracle_commit_path on the equivalent contiguous caches,
    seen through the block table layer by layer, and (2) a direct numpy scatter."""
    rng = np.random.default_rng(31)
    Ly, B, N, Hkv, D, S, ps, F = 3, 3, 9, 2, 8, 48, 16, 5
    cl = np.array([20, 33, 0], dtype=np.int32)
    kc = rng.standard_normal((Ly, B, Hkv, S, D)).astype(np.float32)
    vc = rng.standard_normal((Ly, B, Hkv, S, D)).astype(np.float32)
    for b in range(B):
        kc[:, b, :, cl[b]:] = 0
        vc[:, b, :, cl[b]:] = 0
    max_blocks = S // ps
    num_pages = B * max_blocks + 4
    bt = rng.permutation(num_pages)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
    kp = rng.standard_normal((Ly, num_pages, Hkv, ps, D)).astype(np.float32)
    vp = rng.standard_normal((Ly, num_pages, Hkv, ps, D)).astype(np.float32)
    for l in range(Ly):
        for b in range(B):
            for j in range(S):
                kp[l, bt[b, j // ps], :, j % ps] = kc[l, b, :, j]
                vp[l, bt[b, j // ps], :, j % ps] = vc[l, b, :, j]
    kp0, vp0 = kp.copy(), vp.copy()
    kt = rng.standard_normal((Ly, B, N, Hkv, D)).astype(np.float32)
    vt = rng.standard_normal((Ly, B, N, Hkv, D)).astype(np.float32)
    feats = rng.standard_normal((B, N, F)).astype(np.float32)
    path = np.array([[0, 2, 5, -1], [0, -1, -1, -1], [0, 1, 3, 7]], dtype=np.int32)
    alen = np.array([2, 0, 3], dtype=np.int32)
    fo1 = np.full((B, 4, F), -7.0, dtype=np.float32)
    fo2 = fo1.copy()
    kc2, vc2, cl2 = kc.copy(), vc.copy(), cl.copy()
    d1, s1 = O.commit_path(kt, vt, kc2, vc2, cl2, path, alen, feats, fo1)
    clp = cl.copy()
    d2, s2 = O.commit_path_paged(kt, vt, kp, vp, bt, clp, path, alen, feats, fo2)
    assert np.array_equal(d1, d2) and np.array_equal(s1, s2) and np.array_equal(cl2, clp) and np.array_equal(fo1, fo2)
    for l in range(Ly):
        gk, st = O.paged_gather(kp[l], bt, clp, S)
        gv, _ = O.paged_gather(vp[l], bt, clp, S)
        assert (st == 0).all() and np.array_equal(gk, kc2[l]) and np.array_equal(gv, vc2[l])
    # direct numpy scatter of the same rows; every other byte of the pools untouched
    ke, ve = kp0.copy(), vp0.copy()
    for b in range(B):
        for k in range(alen[b] + 1):
            j = cl[b] + k
            ke[:, bt[b, j // ps], :, j % ps] = kt[:, b, path[b, k]]
            ve[:, bt[b, j // ps], :, j % ps] = vt[:, b, path[b, k]]
    assert np.array_equal(kp, ke) and np.array_equal(vp, ve)
    # a bad page id flags the sequence and leaves it alone in every layer
    bt_bad = bt.copy()
    bt_bad[2, 0] = -1
    kq, vq, clq = kp0.copy(), vp0.copy(), cl.copy()
    d3, s3 = O.commit_path_paged(kt, vt, kq, vq, bt_bad, clq, path, alen)
    assert s3.tolist() == [0, 0, 2] and clq.tolist() == [23, 34, 0] and (d3[2] == -1).all()
    for l in range(Ly):
        for pg in bt[2]:
            assert np.array_equal(kq[l, pg], kp0[l, pg])
