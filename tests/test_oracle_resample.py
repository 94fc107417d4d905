"""Pins of the oracle's sibling-sequential rule with the correction token (Sec. 2,
speculative-sampling paragraph; Sec. 3.2, second equation).  CPU only."""
import os

import numpy as np
import pytest
from scipy.stats import chi2

from oracle import s4c_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def logp(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def read_examples():
    ex = []
    fl = lambda s: [float(x) for x in s.split()]
    ints = lambda s: [int(x) for x in s.split()]
    for line in open(os.path.join(GOLD, "resample_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        ex.append(dict(name=f[0], pt0=fl(f[1]), q0=fl(f[2]), pt1=fl(f[3]), pt2=fl(f[4]), tok=ints(f[5]),
                       u=fl(f[6]), ur=float(f[7]), path=ints(f[8]), bonus=int(f[9])))
    return ex


@pytest.mark.parametrize("ex", read_examples(), ids=lambda e: e["name"])
def test_hand_examples(ex):
    logits = np.stack([logp(ex["pt0"]), logp(ex["pt1"]), logp(ex["pt2"])])[None]
    q = np.zeros((1, 3, 4), dtype=np.float32)
    q[0, 0] = ex["q0"]
    r = O.accept_resample(logits, q, np.array([[-1, 0, 0]]), np.array([[9, ex["tok"][0], ex["tok"][1]]]),
                          np.array([[0.0] + ex["u"]], dtype=np.float32), np.array([ex["ur"]], dtype=np.float32), max_path=3)
    L = len(ex["path"]) - 1
    assert r["accept_len"][0] == L and r["status"][0] == 0
    assert list(r["path"][0]) == ex["path"] + [-1] * (3 - len(ex["path"]))
    want_tok = [ex["tok"][n - 1] for n in ex["path"][1:]]
    assert list(r["accepted_tokens"][0]) == want_tok + [-1] * (3 - len(want_tok))
    assert r["bonus_token"][0] == ex["bonus"]


def _dirichlet_rows(rng, n, V, conc):
    p = rng.dirichlet(np.full(V, conc), size=n)
    return p / p.sum(-1, keepdims=True)


def _chi2_ok(counts, probs, alpha=1e-6):
    n = counts.sum()
    exp = probs * n
    stat = ((counts - exp) ** 2 / exp).sum()
    return stat < chi2.ppf(1 - alpha, len(probs) - 1), stat


@pytest.mark.parametrize("k", [1, 2, 4])
def test_first_emitted_token_follows_the_target(k):
    """The guarantee the rule exists for: with k candidate tokens drawn independently from the
    draft distribution, the token emitted at the root (the accepted candidate, or the
    correction token when all are rejected) is distributed exactly as the target."""
    rng = np.random.default_rng(100 + k)
    V, B = 6, 400_000
    pt = _dirichlet_rows(rng, 1, V, 0.8)[0]
    q = _dirichlet_rows(rng, 1, V, 0.8)[0]
    N = 1 + k
    logits = np.broadcast_to(logp(pt), (B, N, V)).copy()
    dp = np.zeros((B, N, V), dtype=np.float32)
    dp[:, 0] = q.astype(np.float32)
    parent = np.tile(np.array([-1] + [0] * k, dtype=np.int32), (B, 1))
    tokens = np.zeros((B, N), dtype=np.int32)
    tokens[:, 1:] = rng.choice(V, size=(B, k), p=q)
    u = rng.random((B, N), dtype=np.float32)
    ur = rng.random(B, dtype=np.float32)
    r = O.accept_resample(logits, dp, parent, tokens, u, ur, max_path=2)
    first = np.where(r["accept_len"] > 0, r["accepted_tokens"][:, 0], r["bonus_token"])
    ok, stat = _chi2_ok(np.bincount(first, minlength=V).astype(np.float64), pt)
    assert ok, stat
    # and the acceptance rate of the first candidate is sum_x min(pt, q)
    rate = (r["path"][:, 1] == 1).mean()
    assert abs(rate - np.minimum(pt, q).sum()) < 5 * np.sqrt(0.25 / B)


def test_second_level_follows_its_own_target_row():
    """Two levels: the token emitted after an accepted first-level node c follows row c."""
    rng = np.random.default_rng(7)
    V, B = 5, 400_000
    # root 0 -> nodes 1, 2; node 1 -> 3, 4; node 2 -> 5, 6
    parent1 = np.array([-1, 0, 0, 1, 1, 2, 2], dtype=np.int32)
    N = len(parent1)
    pt = _dirichlet_rows(rng, N, V, 1.0)
    q = _dirichlet_rows(rng, N, V, 1.0)
    logits = np.broadcast_to(logp(pt), (B, N, V)).copy()
    dp = np.broadcast_to(q.astype(np.float32), (B, N, V)).copy()
    parent = np.tile(parent1, (B, 1))
    tokens = np.zeros((B, N), dtype=np.int32)
    for c in range(1, N):
        tokens[:, c] = rng.choice(V, size=B, p=q[parent1[c]])
    u = rng.random((B, N), dtype=np.float32)
    ur = rng.random(B, dtype=np.float32)
    r = O.accept_resample(logits, dp, parent, tokens, u, ur, max_path=3)
    L = r["accept_len"]
    first = np.where(L > 0, r["accepted_tokens"][:, 0], r["bonus_token"])
    ok, stat = _chi2_ok(np.bincount(first, minlength=V).astype(np.float64), pt[0])
    assert ok, stat
    for c in (1, 2):
        sel = r["path"][:, 1] == c
        assert sel.sum() > 20_000
        second = np.where(L[sel] > 1, r["accepted_tokens"][sel, 1], r["bonus_token"][sel])
        ok, stat = _chi2_ok(np.bincount(second, minlength=V).astype(np.float64), pt[c])
        assert ok, (c, stat)


def test_equal_draft_and_target_accepts_every_first_child():
    rng = np.random.default_rng(3)
    V = 50
    parent1 = np.array([-1, 0, 0, 1, 1, 3, 3], dtype=np.int32)      # first-child chain 0-1-3-5
    N = len(parent1)
    pt = _dirichlet_rows(rng, N, V, 1.0)
    logits = logp(pt)[None]
    dp = pt.astype(np.float32)[None]
    tokens = rng.integers(0, V, size=(1, N)).astype(np.int32)
    for s in range(20):
        u = (rng.random((1, N)) * 0.99).astype(np.float32)
        r = O.accept_resample(logits, dp, parent1[None], tokens, u, np.array([0.5], np.float32), max_path=4)
        assert list(r["path"][0]) == [0, 1, 3, 5] and r["accept_len"][0] == 3


def test_deterministic_draft():
    """q = point mass at x: accepted iff u < pt(x); otherwise the correction token follows pt with
    x removed, and is never x."""
    V = 8
    rng = np.random.default_rng(11)
    pt = _dirichlet_rows(rng, 1, V, 1.0)[0]
    x = 3
    n = 20_000
    logits = np.broadcast_to(logp(pt), (n, 2, V)).copy()
    dp = np.zeros((n, 2, V), dtype=np.float32)
    dp[:, 0, x] = 1.0
    parent = np.tile(np.array([-1, 0], np.int32), (n, 1))
    tokens = np.tile(np.array([0, x], np.int32), (n, 1))
    u = np.zeros((n, 2), dtype=np.float32)
    u[:, 1] = np.float32(pt[x]) * 1.001          # just above the threshold: always rejected
    ur = ((np.arange(n) + 0.5) / n).astype(np.float32)
    r = O.accept_resample(logits, dp, parent, tokens, u, ur, max_path=2)
    assert (r["accept_len"] == 0).all() and (r["bonus_token"] != x).all()
    want = pt.copy()
    want[x] = 0
    want /= want.sum()
    got = np.bincount(r["bonus_token"], minlength=V) / n
    assert np.abs(got - want).max() < 2.0 / n * V          # a regular grid of u_r: only edge effects
    u[:, 1] = np.float32(pt[x]) * 0.999
    r = O.accept_resample(logits, dp, parent, tokens, u, ur, max_path=2)
    assert (r["accept_len"] == 1).all()


def test_inverse_cdf_on_a_single_node():
    """N = 1: the bonus token is the inverse CDF of the root's target row."""
    V = 7
    pt = np.array([0.05, 0.2, 0.0001, 0.3, 0.25, 0.1, 0.0999])
    n = 100_000
    logits = np.broadcast_to(logp(pt), (n, 1, V)).copy()
    ur = ((np.arange(n) + 0.5) / n).astype(np.float32)
    r = O.accept_resample(logits, np.zeros((n, 1, V), np.float32), np.full((n, 1), -1, np.int32),
                          np.zeros((n, 1), np.int32), np.zeros((n, 1), np.float32), ur, max_path=1)
    want = np.searchsorted(np.cumsum(pt / pt.sum()), ur.astype(np.float64), side="right")
    edge = r["margin_sample"] < 1e-6
    assert (r["bonus_token"][~edge] == want[~edge]).all() and edge.sum() < 10
    assert (r["accept_len"] == 0).all()
    assert r["bonus_token"][0] == 0 and r["bonus_token"][-1] == V - 1


def test_chain_agrees_with_the_per_node_rule():
    """On a chain (one child per node) nothing is carried between siblings, so the accepted
    prefix is that of the per-node rule with p_draft = q[parent][token]."""
    rng = np.random.default_rng(5)
    for case in range(40):
        N, V = int(rng.integers(2, 9)), int(rng.integers(3, 40))
        parent = np.arange(-1, N - 1, dtype=np.int32)[None]
        logits = (2 * rng.standard_normal((1, N, V))).astype(np.float32)
        q = _dirichlet_rows(rng, N, V, 0.7).astype(np.float32)[None]
        tokens = rng.integers(0, V, size=(1, N)).astype(np.int32)
        u = rng.random((1, N), dtype=np.float32)
        pdraft = np.zeros((1, N), dtype=np.float32)
        for i in range(1, N):
            pdraft[0, i] = q[0, i - 1, tokens[0, i]]
        a = O.accept_path(logits, parent, tokens, "stochastic", N, pdraft, u, 1.0)
        b = O.accept_resample(logits, q, parent, tokens, u, np.array([0.5], np.float32), N, 1.0)
        assert a["accept_len"][0] == b["accept_len"][0]
        assert (a["path"] == b["path"]).all() and (a["accepted_tokens"] == b["accepted_tokens"]).all()


def test_temperature_and_margins():
    V = 4
    lg = np.array([[[2.0, 1.0, 0.0, -1.0], [0, 0, 0, 0]]], dtype=np.float32)
    q = np.zeros((1, 2, V), np.float32)
    q[0, 0] = [0.25, 0.25, 0.25, 0.25]
    pt_T2 = np.exp(lg[0, 0] / 2.0) / np.exp(lg[0, 0] / 2.0).sum()
    thr = pt_T2[2] / 0.25                                   # token 2: below 1 at T = 2
    assert thr < 1
    for du, want in ((-1e-3, 1), (+1e-3, 0)):
        u = np.array([[0, thr + du]], np.float32)
        r = O.accept_resample(lg, q, np.array([[-1, 0]]), np.array([[0, 2]]), u, np.array([0.1], np.float32), 2, 2.0)
        assert r["accept_len"][0] == want
        assert 0.5e-3 < r["margin_accept"][0] * 1.0 < 2e-3 / thr


def test_equality_rejects():
    """u * q(x) == r(x) exactly (equal logits over 4 tokens: r = 1/4; q(x) = 1/2, u = 1/2): strict test fails."""
    lg = np.zeros((1, 2, 4), np.float32)
    q = np.zeros((1, 2, 4), np.float32)
    q[0, 0] = [0.5, 0.5, 0, 0]
    for uu, want in ((0.5, 0), (0.49999997, 1)):
        r = O.accept_resample(lg, q, np.array([[-1, 0]]), np.array([[0, 1]]), np.array([[0, uu]], np.float32),
                              np.array([0.1], np.float32), 2)
        assert r["accept_len"][0] == want


def test_bad_tree_and_bad_token():
    V = 5
    lg = np.zeros((2, 3, V), np.float32)
    q = np.full((2, 3, V), 0.2, np.float32)
    parent = np.array([[-1, 0, 0], [-1, 2, 0]], np.int32)       # second tree: parent after child
    tokens = np.array([[0, 77, 1], [0, 1, 1]], np.int32)         # first tree: node 1 holds no token id
    u = np.full((2, 3), 0.5, np.float32)
    r = O.accept_resample(lg, q, parent, tokens, u, np.array([0.5, 0.5], np.float32), 3)
    assert r["status"][1] == 1 and r["accept_len"][1] == 0 and r["bonus_token"][1] == -1
    assert list(r["path"][1]) == [0, -1, -1]
    # node 1 is skipped with the residual untouched; node 2 (token 1): 0.5 * 0.2 < 0.2 -> accepted
    assert r["status"][0] == 0 and list(r["path"][0]) == [0, 2, -1]
