"""HIP-graph replay of the entry points beyond the three-call step: s4c_build_tree, s4c_draft_linear,
s4c_accept_resample (whose slot array is cleared by a fill kernel, not a memset node) and
s4c_commit_path with feature rows.  The sequence is captured once and replayed several times with
eager work and synchronisations in between; every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.device import np_to_torch
from paper_2506_14158_amd.verify import TreeVerifier
from tests.util import resample_inputs_with_margin, to_device
from tests.test_gpu_build_tree import counts_of

pytestmark = pytest.mark.gpu


def test_drafter_side_calls_replay_from_a_hip_graph():
    cfg = synth.scaled(synth.CONFIGS[3], name="graph-next", B=3, V=40000, index=0)       # V large enough for workgroup teams
    par = synth.make_parent(cfg)
    ac, r = resample_inputs_with_margin(cfg, par, O)
    ac2 = synth.make_accept_inputs(cfg, par, keep_draft_logits=True)
    d = to_device(cfg, par, None, ac)
    N, levels, Bn = cfg.N, cfg.levels, cfg.B
    tv = TreeVerifier(Bn, N, 1, 1, 64, 1, cfg.V, d["logits"].dtype, levels, 0)
    # tree construction inputs / outputs
    nchild = torch.from_numpy(counts_of(par)).cuda()
    kmax = int(nchild.max())
    dl = np_to_torch(ac2.draft_logits)
    root = torch.from_numpy(ac2.tokens[:, 0].copy()).cuda()
    bt_ws = B.alloc_workspace(B.s4c_build_tree_workspace_size(Bn, N, cfg.V))
    o_par, o_tok = torch.empty_like(d["parent"]), torch.empty_like(d["parent"])
    o_pd = torch.empty(Bn, N, dtype=torch.float32, device="cuda")
    # projection
    g = torch.Generator(device="cuda").manual_seed(5)
    T, H = Bn * N, 256
    e, f = (torch.randn(T, H, device="cuda", generator=g).bfloat16() for _ in range(2))
    W = (torch.randn(H, 2 * H, device="cuda", generator=g) / (2 * H) ** 0.5).bfloat16()
    h_out = torch.empty(T, H, dtype=torch.bfloat16, device="cuda")
    dl_ws = B.alloc_workspace(B.s4c_draft_linear_workspace_size(T, H, H))      # None above 128 tokens
    # the same projection on one sequence's tokens (<= 128: the weight-streaming kernel and its workspace)
    h_small = torch.empty(N, H, dtype=torch.bfloat16, device="cuda")
    dl_ws_small = B.alloc_workspace(B.s4c_draft_linear_workspace_size(N, H, H))
    # commit: 3 layers + feature rows
    Ly, Hkv, D, P = 3, 2, 128, 100
    S_cap = P + levels
    mk = lambda *s: torch.randn(*s, device="cuda", generator=g).bfloat16()
    kt, vt = mk(Ly, Bn, N, Hkv, D), mk(Ly, Bn, N, Hkv, D)
    kc0, vc0 = mk(Ly, Bn, Hkv, S_cap, D), mk(Ly, Bn, Hkv, S_cap, D)
    kc, vc = kc0.clone(), vc0.clone()
    cl0 = torch.full((Bn,), P, dtype=torch.int32, device="cuda")
    cl = cl0.clone()
    feats = mk(Bn, N, H)
    fout = torch.zeros(Bn, levels, H, dtype=torch.bfloat16, device="cuda")

    def calls():
        B.s4c_build_tree(dl, nchild, root, kmax, o_par, o_tok, o_pd, bt_ws, cfg.temperature)
        B.s4c_draft_linear(e, f, W, h_out, None, dl_ws)
        B.s4c_draft_linear(e[:N], f[:N], W, h_small, None, dl_ws_small)
        tv.accept_resample(d["logits"], d["draft_probs"], d["parent"], d["tokens"], d["uniforms"], d["u_resample"],
                           cfg.temperature)
        tv.commit_path(kt, vt, kc, vc, cl, feats, fout)

    outs = lambda: (o_par, o_tok, o_pd, h_out, h_small, tv.path, tv.accept_len, tv.bonus_token, kc, vc, cl, fout)
    bits = lambda t: t.view(torch.int16) if t.dtype == torch.bfloat16 else t

    def reset():
        kc.copy_(kc0); vc.copy_(vc0); cl.copy_(cl0)
        for t in (o_par, o_tok, tv.path, tv.accept_len, tv.bonus_token):
            t.fill_(-9)
        o_pd.fill_(-1.0); h_out.zero_(); h_small.zero_(); fout.zero_()

    calls()                                  # eager once: allocates the verifier's slot workspace, gives the reference
    torch.cuda.synchronize()
    reset()
    calls()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs()]
    assert np.array_equal(tv.path.cpu().numpy(), r["path"]) and np.array_equal(o_par.cpu().numpy(), par)   # and the eager run is right
    side = torch.cuda.Stream()
    gr = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(gr, stream=side):
            calls()
    for rep in range(3):
        reset()                              # eager work between replays
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        for a_, b_ in zip(outs(), ref):
            assert torch.equal(bits(a_), bits(b_)), rep
