"""GPU-vs-oracle parity of s4c_accept_resample (sibling-sequential rule with the correction
token) through the C ABI: paths, accepted tokens and the correction token bit-exact."""
import os

import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.verify import TreeVerifier
from tests.util import resample_inputs_with_margin, to_device, RESAMPLE_MARGIN_MIN
from tests.test_oracle_resample import read_examples, logp

pytestmark = pytest.mark.gpu
C = synth.CONFIGS


def run(cfg, par, ac, max_path=None):
    d = to_device(cfg, par, None, ac)
    tv = TreeVerifier(cfg.B, cfg.N, 1, 1, 64, 1, cfg.V, d["logits"].dtype, cfg.levels if max_path is None else max_path, 0)
    for t in (tv.path, tv.accept_len, tv.accepted_tokens, tv.bonus_token, tv.accept_status):
        t.fill_(-7)
    tv.accept_resample(d["logits"], d["draft_probs"], d["parent"], d["tokens"], d["uniforms"], d["u_resample"],
                       cfg.temperature)
    torch.cuda.synchronize()
    return tv


def same(tv, r):
    assert np.array_equal(tv.accept_status.cpu().numpy(), r["status"])
    assert np.array_equal(tv.accept_len.cpu().numpy(), r["accept_len"])
    assert np.array_equal(tv.path.cpu().numpy(), r["path"])
    assert np.array_equal(tv.accepted_tokens.cpu().numpy(), r["accepted_tokens"])
    assert np.array_equal(tv.bonus_token.cpu().numpy(), r["bonus_token"])


def check(cfg):
    par = synth.make_parent(cfg)
    ac, r = resample_inputs_with_margin(cfg, par, O)
    tv = run(cfg, par, ac)
    same(tv, r)
    return r


SMALL = [
    synth.scaled(C[3], name="13b-small", B=3, V=9000, index=0),
    synth.scaled(C[3], name="13b-temp", B=2, V=9000, temperature=0.7, index=0),
    synth.scaled(C[3], name="13b-v-odd", B=3, V=8191 * 3 + 5, index=0),                   # rows not 16-byte aligned
    synth.scaled(C[3], name="13b-v-tiny", B=4, V=130, index=0),                           # one partial block
    synth.scaled(C[5], name="70b-small", B=2, V=20000, index=0),                          # N = 128
    synth.scaled(C[1], name="f32", mode="stochastic", B=4, V=5000, N=31, levels=5, index=0),
    synth.scaled(C[1], name="f32-v-odd", mode="stochastic", B=2, V=1003, N=15, levels=4, index=0),
    synth.scaled(C[3], name="root-only", B=3, V=4000, N=1, levels=1, index=0),
    synth.scaled(C[3], name="13b-v-1m", B=2, V=1_000_003, N=6, levels=3, index=0),        # long, odd rows; 16 workgroups each
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_accept_resample_small(cfg):
    check(cfg)


@pytest.mark.parametrize("idx", [3, 5])
def test_accept_resample_full_size(idx):
    r = check(C[idx])
    print("cfg%d sequential accept_len" % idx, r["accept_len"].tolist(), "correction tokens", r["bonus_token"].tolist())


def test_independent_candidates_many_sequences():
    """Candidates drawn independently from the draft (the setting of the rule's guarantee), small V,
    many rejections and corrections per tree: 2000 sequences against the oracle."""
    rng = np.random.default_rng(21)
    Bn, V = 2000, 48
    par1 = np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 4, 4], dtype=np.int32)
    N = len(par1)
    par = np.tile(par1, (Bn, 1))
    logits = (1.5 * rng.standard_normal((Bn, N, V))).astype(np.float32)
    q = rng.dirichlet(np.full(V, 0.5), size=(Bn, N)).astype(np.float32)
    tokens = np.zeros((Bn, N), dtype=np.int32)
    for c in range(1, N):
        cdf = np.cumsum(q[:, par1[c]].astype(np.float64), axis=1)
        tokens[:, c] = np.minimum((cdf < rng.random((Bn, 1)) * cdf[:, -1:]).sum(1), V - 1)
    u = rng.random((Bn, N), dtype=np.float32)
    ur = rng.random(Bn, dtype=np.float32)
    r = O.accept_resample(logits, q, par, tokens, u, ur, 4)
    good = (r["margin_accept"] > RESAMPLE_MARGIN_MIN) & (r["margin_sample"] > RESAMPLE_MARGIN_MIN)
    assert good.mean() > 0.999
    cfg = synth.scaled(C[1], name="iid", mode="stochastic", B=Bn, N=N, V=V, levels=4, index=0)
    ac = synth.AcceptInputs(logits, tokens, np.zeros((Bn, N), np.float32), u, q, ur)
    tv = run(cfg, par, ac)
    for name in ("accept_len", "bonus_token"):
        assert np.array_equal(getattr(tv, name).cpu().numpy()[good], r[name][good])
    assert np.array_equal(tv.path.cpu().numpy()[good], r["path"][good])
    assert (r["accept_len"] > 0).mean() > 0.3 and (r["accept_len"] == 0).mean() > 0.05


@pytest.mark.parametrize("ex", read_examples(), ids=lambda e: e["name"])
def test_hand_examples_on_the_gpu(ex):
    logits = np.stack([logp(ex["pt0"]), logp(ex["pt1"]), logp(ex["pt2"])])[None]
    q = np.zeros((1, 3, 4), dtype=np.float32)
    q[0, 0] = ex["q0"]
    par = np.array([[-1, 0, 0]], dtype=np.int32)
    tokens = np.array([[9, ex["tok"][0], ex["tok"][1]]], dtype=np.int32)
    cfg = synth.scaled(C[1], name="hand", mode="stochastic", B=1, N=3, V=4, levels=3, index=0)
    ac = synth.AcceptInputs(logits, tokens, np.zeros((1, 3), np.float32), np.array([[0.0] + ex["u"]], np.float32), q,
                            np.array([ex["ur"]], np.float32))
    tv = run(cfg, par, ac)
    assert tv.path.cpu().tolist()[0] == ex["path"] + [-1] * (3 - len(ex["path"]))
    assert int(tv.bonus_token[0]) == ex["bonus"] and int(tv.accept_len[0]) == len(ex["path"]) - 1


def test_equality_rejects_bad_tree_and_bad_token():
    # u * q(x) == r(x) exactly: strict test fails on the GPU as in the oracle
    lg = np.zeros((1, 2, 4), np.float32)
    q = np.zeros((1, 2, 4), np.float32)
    q[0, 0] = [0.5, 0.5, 0, 0]
    cfg = synth.scaled(C[1], name="eq", mode="stochastic", B=1, N=2, V=4, levels=2, index=0)
    for uu, want in ((0.5, 0), (0.49999997, 1)):
        ac = synth.AcceptInputs(lg, np.array([[0, 1]], np.int32), np.zeros((1, 2), np.float32),
                                np.array([[0, uu]], np.float32), q, np.array([0.1], np.float32))
        tv = run(cfg, np.array([[-1, 0]], np.int32), ac)
        assert int(tv.accept_len[0]) == want
    # malformed tree -> flagged; token outside the vocabulary -> skipped
    V = 5
    lg = np.zeros((2, 3, V), np.float32)
    q = np.full((2, 3, V), 0.2, np.float32)
    par = np.array([[-1, 0, 0], [-1, 2, 0]], np.int32)
    tokens = np.array([[0, 77, 1], [0, 1, 1]], np.int32)
    u = np.full((2, 3), 0.5, np.float32)
    ur = np.array([0.5, 0.5], np.float32)
    cfg = synth.scaled(C[1], name="bad", mode="stochastic", B=2, N=3, V=V, levels=3, index=0)
    tv = run(cfg, par, synth.AcceptInputs(lg, tokens, np.zeros((2, 3), np.float32), u, q, ur))
    same(tv, O.accept_resample(lg, q, par, tokens, u, ur, 3))
    assert tv.accept_status.cpu().tolist() == [0, 1]


def test_team_that_cannot_exchange_is_flagged_and_every_kernel_exits(monkeypatch):
    """The bounded wait of the workgroup teams, forced from the host: with zero polls allowed a
    workgroup that does not find all of its team's partial sums at its first look gives up, so no
    team of several workgroups completes.  Every kernel must still exit, and every such sequence
    must come back as the flagged empty result (written by the team's first workgroup alone); the
    next call with the default limit gives the oracle's answer again on the same buffers."""
    cfg = synth.scaled(C[3], name="timeout", B=3, V=40000, index=0)          # teams of 10 workgroups
    par = synth.make_parent(cfg)
    ac, r = resample_inputs_with_margin(cfg, par, O)
    assert B.s4c_accept_resample_workspace_size(cfg.B, cfg.N, cfg.V, cfg.levels) > 0    # teams of more than one workgroup
    d = to_device(cfg, par, None, ac)
    tv = TreeVerifier(cfg.B, cfg.N, 1, 1, 64, 1, cfg.V, d["logits"].dtype, cfg.levels, 0)
    call = lambda: tv.accept_resample(d["logits"], d["draft_probs"], d["parent"], d["tokens"], d["uniforms"],
                                      d["u_resample"], cfg.temperature)
    monkeypatch.setenv("S4C_RESAMPLE_SPIN_LIMIT", "0")
    for rep in range(3):
        for t in (tv.path, tv.accept_len, tv.accepted_tokens, tv.bonus_token, tv.accept_status):
            t.fill_(-7)
        call()
        torch.cuda.synchronize()
        assert tv.accept_status.cpu().tolist() == [B.S4C_SEQ_TIMEOUT] * cfg.B, rep
        assert tv.accept_len.cpu().tolist() == [0] * cfg.B and tv.bonus_token.cpu().tolist() == [-1] * cfg.B
        assert tv.path.cpu().tolist() == [[0] + [-1] * (cfg.levels - 1)] * cfg.B
        assert (tv.accepted_tokens.cpu().numpy() == -1).all()
    monkeypatch.delenv("S4C_RESAMPLE_SPIN_LIMIT")
    call()
    torch.cuda.synchronize()
    same(tv, r)


def test_rejects_bad_arguments():
    t = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    i = lambda *s: torch.zeros(*s, dtype=torch.int32, device="cuda")
    with pytest.raises(B.S4CError):      # temperature must be positive
        B.s4c_accept_resample(t(1, 2, 8), t(1, 2, 8), i(1, 2), i(1, 2), t(1, 2), t(1), 2, i(1, 2), i(1), i(1, 2), i(1),
                              temperature=0.0)
    with pytest.raises(B.S4CError):      # a team of workgroups needs its exchange workspace
        assert B.s4c_accept_resample_workspace_size(2, 3, 40000, 3) > 0
        B.s4c_accept_resample(t(2, 3, 40000), t(2, 3, 40000), i(2, 3), i(2, 3), t(2, 3), t(2), 3, i(2, 3), i(2), i(2, 3),
                              i(2), workspace=None)
    with pytest.raises(B.S4CError):      # more nodes than a tree may hold
        B.s4c_accept_resample(t(1, 129, 8), t(1, 129, 8), i(1, 129), i(1, 129), t(1, 129), t(1), 2, i(1, 2), i(1),
                              i(1, 2), i(1))
