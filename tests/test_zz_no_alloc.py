"""s4c_accept_path_static (the entry point that allocates nothing and takes no workspace) against
s4c_accept_path on the same inputs: every output bit-identical, on two calls in a row that share the
library's fixed scratch, the second with a smaller input.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from tests.util import accept_inputs_with_margin, to_device

pytestmark = pytest.mark.gpu
C = synth.CONFIGS


def _outputs(Bn, max_path):
    i32 = dict(dtype=torch.int32, device="cuda")
    return dict(path=torch.full((Bn, max_path), -7, **i32), accept_len=torch.full((Bn,), -7, **i32),
                accepted_tokens=torch.full((Bn, max_path), -7, **i32), bonus_token=torch.full((Bn,), -7, **i32),
                status=torch.full((Bn,), -7, **i32))


def _prepare(cfg):
    par = synth.make_parent(cfg)
    ac, r = accept_inputs_with_margin(cfg, par, O)
    d = to_device(cfg, par, None, ac)
    ws = B.alloc_workspace(B.s4c_accept_path_workspace_size(cfg.B, cfg.N, cfg.V))
    return cfg, d, r, ws, _outputs(cfg.B, cfg.levels), _outputs(cfg.B, cfg.levels)


def _run(case, static):
    cfg, d, r, ws, o_ws, o_st = case
    mode = B.S4C_GREEDY if cfg.mode == "greedy" else B.S4C_STOCHASTIC
    o = o_st if static else o_ws
    args = (d["logits"], d["parent"], d["tokens"], mode, cfg.levels, o["path"], o["accept_len"], o["accepted_tokens"],
            o["bonus_token"])
    kw = dict(p_draft=d["p_draft"], uniforms=d["uniforms"], temperature=cfg.temperature, status=o["status"])
    if static:
        B.s4c_accept_path_static(*args, **kw)
    else:
        B.s4c_accept_path(*args, ws, **kw)


def _check(case):
    cfg, d, r, ws, o_ws, o_st = case
    for k in o_ws:
        assert torch.equal(o_ws[k], o_st[k]), (cfg.name, k)
    # and both are the oracle's answer
    assert np.array_equal(o_st["path"].cpu().numpy(), r["path"])
    assert np.array_equal(o_st["accept_len"].cpu().numpy(), r["accept_len"])
    assert np.array_equal(o_st["accepted_tokens"].cpu().numpy(), r["accepted_tokens"])
    assert np.array_equal(o_st["bonus_token"].cpu().numpy(), r["bonus_token"])
    assert np.array_equal(o_st["status"].cpu().numpy(), r["status"])


@pytest.mark.parametrize("big,small", [
    (synth.scaled(C[5], name="static-stoch-big", B=4, V=50000, index=0),
     synth.scaled(C[3], name="static-stoch-small", B=2, V=9000, index=0)),
    (synth.scaled(C[4], name="static-greedy-big", B=3, V=70001, index=0),
     synth.scaled(C[1], name="static-greedy-small", B=2, index=0)),
], ids=["stochastic", "greedy"])
def test_static_scratch_entry_matches_workspace_entry(big, small):
    first, second = _prepare(big), _prepare(small)
    for case in (first, second):
        _run(case, static=False)
    torch.cuda.synchronize()
    _run(first, static=True)                    # also the first call on this GPU: looks up the scratch address
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    _run(second, static=True)                   # smaller input over the scratch the first call left behind
    _run(first, static=True)                    # and the larger one again, back to back on one stream
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before      # no device memory was taken by the calls
    _check(second)
    _check(first)
