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
