"""Pins of the oracle's candidate-tree construction (Sec. 3.2: top-1 continuation first, next most
probable tokens beside it).  CPU only."""
import os

import numpy as np
from scipy.special import softmax

from oracle import s4c_oracle as O
from paper_2506_14158_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_fig3_layout():
    """Child counts of the Fig. 3 example (2 after the root, 1 after each of them, 2 after each of
    those) must give the hand-numbered parent array of the golden file."""
    want = None
    for line in open(os.path.join(GOLD, "fig3_tree.txt")):
        if line.startswith("parent"):
            want = [int(x) for x in line.split()[1:]]
    nchild = np.array([[2, 1, 1, 2, 2, 0, 0, 0, 0]], dtype=np.int32)
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((1, 9, 50)).astype(np.float32)
    r = O.build_tree(lg, nchild, np.array([7]), kmax=2)
    assert r["parent"][0].tolist() == want and r["status"][0] == 0
    assert r["level"][0].tolist() == [0, 1, 1, 2, 2, 3, 3, 3, 3]
    assert r["tokens"][0, 0] == 7 and r["p_draft"][0, 0] == 0


def test_children_are_the_top_k_tokens_with_their_probabilities():
    rng = np.random.default_rng(1)
    B, N, V, kmax = 3, 12, 300, 4
    for dtype in ("f32", "bf16-ties"):
        lg = (2 * rng.standard_normal((B, N, V))).astype(np.float32)
        if dtype != "f32":
            lg = synth.f32_to_bf16_bits(np.round(lg))            # integer logits: many equal values
        nchild = np.zeros((B, N), dtype=np.int32)
        nchild[:, 0], nchild[:, 1], nchild[:, 2], nchild[:, 3], nchild[:, 5] = 4, 3, 2, 1, 1
        T = 0.8
        r = O.build_tree(lg, nchild, np.arange(B), kmax, temperature=T)
        assert (r["status"] == 0).all()
        f = lg if dtype == "f32" else synth.bf16_bits_to_f32(lg)
        for b in range(B):
            nxt = 1
            for i in range(N):
                k = nchild[b, i]
                if not k:
                    continue
                order = np.lexsort((np.arange(V), -f[b, i].astype(np.float64)))[:k]   # value desc, id asc
                p = softmax(f[b, i].astype(np.float64) / T)
                kids = list(range(nxt, nxt + k))
                nxt += k
                assert r["tokens"][b, kids].tolist() == order.tolist()
                assert (r["parent"][b, kids] == i).all()
                np.testing.assert_allclose(r["p_draft"][b, kids], p[order], rtol=2e-7)
            assert nxt == N


def test_reproduces_the_synthetic_workload_trees():
    """The seeded generator builds its stochastic trees in numpy (BFS-labelled, children = the
    draft's top-k in decreasing probability); the oracle must rebuild them from the draft logits
    and the child counts alone."""
    cfg = synth.scaled(synth.CONFIGS[3], B=3, V=4000, index=0)
    par = synth.make_parent(cfg)
    ac = synth.make_accept_inputs(cfg, par, keep_draft_logits=True)
    nchild = np.zeros_like(par)
    for b in range(cfg.B):
        for i in range(1, cfg.N):
            nchild[b, par[b, i]] += 1
    r = O.build_tree(ac.draft_logits, nchild, ac.tokens[:, 0], kmax=int(nchild.max()), temperature=1.0)
    assert np.array_equal(r["parent"], par)
    assert np.array_equal(r["tokens"], ac.tokens)
    np.testing.assert_allclose(r["p_draft"], ac.p_draft, rtol=3e-7)
    assert np.array_equal(r["level"], np.stack([synth.levels_of(par[b]) for b in range(cfg.B)]))


def test_invalid_child_counts_and_tiny_vocabulary():
    lg = np.zeros((4, 4, 2), np.float32)
    lg[:, :, 1] = 1.0
    nchild = np.array([[3, 0, 0, 0],       # fine: three children, but only two tokens exist
                       [1, 0, 1, 0],       # node 2 is a parent before it exists
                       [2, 2, 0, 0],       # 5 nodes described, N = 4
                       [4, 0, 0, 0]],      # more than kmax
                      dtype=np.int32)
    r = O.build_tree(lg, nchild, np.array([5, 5, 5, 5]), kmax=3)
    assert r["status"].tolist() == [0, 1, 1, 1]
    assert r["tokens"][0].tolist() == [5, 1, 0, -1] and r["parent"][0].tolist() == [-1, 0, 0, 0]
    assert r["p_draft"][0, 3] == 0
    for b in (1, 2, 3):
        assert r["parent"][b].tolist() == [-1] * 4 and r["tokens"][b].tolist() == [5, -1, -1, -1]
