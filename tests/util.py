"""Shared test plumbing: error metrics and well-conditioned stochastic workloads."""
import numpy as np
import torch

from paper_2506_14158_amd import synth
from paper_2506_14158_amd.device import np_to_torch, to_device  # noqa: F401


def attn_errors(out_t: torch.Tensor, ref: np.ndarray):
    """(max |g - o|, max over rows of ||g - o||_2 / ||o||_2); a row is one (b, node, head) vector."""
    g = out_t.detach().float().cpu().numpy().astype(np.float64).reshape(-1, ref.shape[-1])
    o = ref.reshape(-1, ref.shape[-1])
    amax = float(np.abs(g - o).max()) if g.size else 0.0
    den = np.linalg.norm(o, axis=1)
    num = np.linalg.norm(g - o, axis=1)
    rel = float((num / np.maximum(den, 1e-30)).max()) if g.size else 0.0
    return amax, rel


MARGIN_MIN = 2e-5   # relative gap |u*pd - pt| / max(..) below which fp32 and fp64 may disagree


def accept_inputs_with_margin(cfg, parent, oracle_mod, max_tries=8):
    """Stochastic workloads: re-draw (seed + 1000 k) until every tested node's decision is at
    least MARGIN_MIN away from equality, so that fp32 (GPU) and fp64 (oracle) must agree."""
    for k in range(max_tries):
        ac = synth.make_accept_inputs(cfg, parent, seed=cfg.seed() + 1000 * k)
        r = oracle_mod.accept_path(ac.logits, parent, ac.tokens, cfg.mode, cfg.levels, ac.p_draft, ac.uniforms,
                                   cfg.temperature)
        if cfg.mode == "greedy" or float(r["margin"].min()) > MARGIN_MIN:
            return ac, r
    raise RuntimeError("no well-conditioned seed found")


RESAMPLE_MARGIN_MIN = 1e-9   # fp64 on both sides: sums of <= 2^21 terms differ by ~1e-13 relative


def resample_inputs_with_margin(cfg, parent, oracle_mod, max_tries=8):
    """Sequential rule with the correction token: the GPU and the oracle both work in fp64 but add
    in different orders, so a decision closer to equality than RESAMPLE_MARGIN_MIN (relative) is
    not comparable.  The correction token's uniform is re-drawn for such a case (expected about
    once in 10^4 sequences); an accept test that close fails the workload."""
    ac = synth.make_accept_inputs(cfg, parent, full_draft=True)
    for k in range(max_tries):
        r = oracle_mod.accept_resample(ac.logits, ac.draft_probs, parent, ac.tokens, ac.uniforms, ac.u_resample,
                                       cfg.levels, cfg.temperature)
        assert float(r["margin_accept"].min()) > RESAMPLE_MARGIN_MIN
        if float(r["margin_sample"][r["status"] == 0].min(initial=1.0)) > RESAMPLE_MARGIN_MIN:
            return ac, r
        ac.u_resample = synth.draw_u_resample(cfg.seed(), cfg.B, attempt=k + 1)
    raise RuntimeError("no well-conditioned correction-token uniforms found")
