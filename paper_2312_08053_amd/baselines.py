"""The allocators the paper compares in its Kimad+ experiment (Section 4.3, Fig. "Kimad+"), run
through the library's calls: argument marshalling only, every number comes from the C ABI.

    kimad_plus      per-layer K from the knapsack allocation over the ratio grid (Section 3.2)
    uniform_ratio   one ratio rho = P / d for every layer, K_i = ceil(rho * d_i)  ("Kimad"): kimad_uniform_sizes
    whole_model     TopK with K = min(P, d) over the concatenation of all layers (the paper's "optimal" line):
                    the payload of a one-layer plan over the flat buffer, split by layer with
                    kimad_payload_layer_counts

Each entry reports the pairs sent and the squared l2 error of what is dropped, per layer (kimad_error_at on the
per-layer plan) and in total (summed on the device).
"""
from __future__ import annotations

from typing import Sequence

from .binding import Plan, kimad_payload_layer_counts, kimad_uniform_sizes


def allocator_errors(g, h, sizes: Sequence[int], ratios: Sequence[float], budget_bytes: int,
                     pair_bytes: int = 8, D: int = 0, per_layer: bool = False) -> dict:
    """g, h: flat fp32 CUDA tensors holding the layers back to back.  Leaves h untouched."""
    import torch
    L = len(sizes)
    out = {}
    plan = Plan(g, h, sizes, ratios, pair_bytes=pair_bytes, D=D, max_budget_bytes=budget_bytes, capacity_pairs=1)
    plan.profile(budget_hint_bytes=budget_bytes)
    plan.allocate(budget_bytes)
    status = int(plan.status[0].item())
    if status == 0:
        E = plan.error_at(plan.K)
        out["kimad_plus"] = {"status": 0, "error": float(E.sum().item()), "pairs": int(plan.offsets[-1].item())}
        if per_layer:
            out["kimad_plus"]["layer_pairs"] = plan.K.cpu().tolist()
            out["kimad_plus"]["layer_errors"] = E.cpu().tolist()
    else:
        out["kimad_plus"] = {"status": status, "error": None, "pairs": 0}

    Ku, P = kimad_uniform_sizes(sizes, budget_bytes, pair_bytes)
    if P > 0:
        Ku_dev = torch.tensor(Ku, dtype=torch.int64, device=g.device)
        Eu = plan.error_at(Ku_dev)
        out["uniform_ratio"] = {"error": float(Eu.sum().item()), "pairs": int(Ku_dev.sum().item())}
        # whole model: one layer spanning the flat buffer, on a copy of the estimator (the selection updates it)
        d = int(g.numel())
        h2 = h.clone()
        whole = Plan(g, h2, [d], [1.0], pair_bytes=pair_bytes, D=1000, capacity_pairs=P)   # (its allocation tables are not used: kept small)
        Kw = torch.tensor([P], dtype=torch.int64, device=g.device)
        offw = torch.tensor([0, P], dtype=torch.int64, device=g.device)
        whole.compress_ef(Kw, offw, reuse_profile=False)
        assert int(whole.status[1].item()) == 0
        starts = torch.zeros(L + 1, dtype=torch.int64, device=g.device)
        starts[1:] = torch.cumsum(torch.tensor([int(s) for s in sizes], dtype=torch.int64, device=g.device), 0)
        counts = torch.empty(L, dtype=torch.int64, device=g.device)
        kimad_payload_layer_counts(whole.idx, P, starts, counts)
        Ew = plan.error_at(counts)
        out["whole_model"] = {"error": float(Ew.sum().item()), "pairs": int(counts.sum().item())}
        if per_layer:
            out["uniform_ratio"]["layer_pairs"] = Ku
            out["uniform_ratio"]["layer_errors"] = Eu.cpu().tolist()
            out["whole_model"]["layer_pairs"] = counts.cpu().tolist()
            out["whole_model"]["layer_errors"] = Ew.cpu().tolist()
        del whole, h2
    return out
