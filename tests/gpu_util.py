"""Host<->device plumbing for the GPU tests (no arithmetic of the method)."""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si
from paper_2604_13349_amd import binding as B


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def run_fused(cfg: si.RelayConfig, K, V, Q, budgets=None, budget=None, rank=None, max_budget=None, layerwise=False, variant=None, n_tokens=None, sink=None):
    """K, V, Q numpy (I/O dtype).  Returns dict of numpy outputs."""
    Kd, Vd, Qd = to_dev(K, cfg.dtype), to_dev(V, cfg.dtype), to_dev(Q, cfg.dtype)
    rank = cfg.rank if rank is None else rank
    kw = dict(rank=rank, want_scores=True, want_delta=True, want_diag=True, layerwise=layerwise, variant=variant, n_tokens=n_tokens, sink=sink)
    if budgets is not None:
        o = B.compress_relay(Kd, Vd, Qd, budgets=np.asarray(budgets).reshape(-1), max_budget=max_budget, **kw)
    else:
        o = B.compress_relay(Kd, Vd, Qd, budget=budget, max_budget=max_budget, **kw)
    torch.cuda.synchronize()
    return {
        "K_out": to_host(o["K_out"], cfg.dtype), "V_out": to_host(o["V_out"], cfg.dtype),
        "idx": o["idx"].cpu().numpy(), "n_keep": o["n_keep"].cpu().numpy(),
        "scores": o["scores"].cpu().numpy(), "delta": o["delta"].cpu().numpy(), "diag": B.diag_to_numpy(o["diag"]),
    }
