"""Move a numpy workload (see synth) into device tensors; bf16 bit patterns become bfloat16."""
import numpy as np
import torch


def np_to_torch(a: np.ndarray, device="cuda") -> torch.Tensor:
    t = torch.from_numpy(a)
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(device)


def to_device(cfg, parent, at=None, ac=None, device="cuda"):
    d = {"parent": torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).to(device)}
    if at is not None:
        for k in ("q", "k_tree", "v_tree", "k_cache", "v_cache"):
            d[k] = np_to_torch(getattr(at, k), device)
        d["cache_len"] = torch.from_numpy(at.cache_len.copy()).to(device)
    if ac is not None:
        d["logits"] = np_to_torch(ac.logits, device)
        d["tokens"] = torch.from_numpy(ac.tokens).to(device)
        d["p_draft"] = torch.from_numpy(ac.p_draft).to(device)
        d["uniforms"] = torch.from_numpy(ac.uniforms).to(device)
        if ac.draft_probs is not None:
            d["draft_probs"] = torch.from_numpy(ac.draft_probs).to(device)
            d["u_resample"] = torch.from_numpy(ac.u_resample).to(device)
    return d
