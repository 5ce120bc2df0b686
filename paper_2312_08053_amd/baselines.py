"""The allocators the paper compares in its Kimad+ experiment (Section 4.3, Fig. "Kimad+"), run
through the same library calls: argument marshalling only, every number comes from the kernels.

    kimad_plus      per-layer K from the knapsack allocation over the ratio grid (Section 3.2)
    uniform_ratio   one ratio rho = P / d for every layer, K_i = ceil(rho * d_i)  ("Kimad")
    whole_model     TopK with K = P over the concatenation of all layers (the paper's "optimal" line)

Each entry reports the squared l2 error of what is dropped and the pairs sent.  The uniform and the
whole-model baselines are plans with a one-ratio grid (and, for the latter, a single layer spanning
the flat buffer), so their errors are rows of `kimad_profile` as well.
"""
from __future__ import annotations

from typing import Sequence

from .binding import Plan


def allocator_errors(g, h, sizes: Sequence[int], ratios: Sequence[float], budget_bytes: int,
                     pair_bytes: int = 8, D: int = 0) -> dict:
    """g, h: flat fp32 CUDA tensors holding the layers back to back.  Leaves h untouched."""
    import torch
    d = int(sum(int(s) for s in sizes))
    P = int(budget_bytes) // int(pair_bytes)
    out = {}

    plan = Plan(g, h, sizes, ratios, pair_bytes=pair_bytes, D=D, max_budget_bytes=budget_bytes)
    plan.profile(budget_hint_bytes=budget_bytes)
    plan.allocate(budget_bytes)
    torch.cuda.synchronize()
    status = int(plan.status[0].item())
    E = plan.err_table.cpu().reshape(len(sizes), -1)
    j = plan.j.cpu().tolist()
    out["kimad_plus"] = {"status": status,
                         "error": float(sum(E[i, j[i]].item() for i in range(len(sizes)))) if status == 0 else None,
                         "pairs": int(plan.offsets[-1].item()) if status == 0 else 0}
    del plan

    rho = min(1.0, P / d)
    if rho > 0.0:
        uni = Plan(g, h, sizes, [rho], pair_bytes=pair_bytes)
        uni.profile()
        torch.cuda.synchronize()
        out["uniform_ratio"] = {"ratio": rho, "error": float(uni.err_table.cpu().sum().item()),
                                "pairs": int(uni.grid_sizes().sum())}
        del uni
        whole = Plan(g, h, [d], [rho], pair_bytes=pair_bytes)
        whole.profile()
        torch.cuda.synchronize()
        out["whole_model"] = {"error": float(whole.err_table.cpu()[0].item()), "pairs": int(whole.grid_sizes()[0, 0])}
        del whole
    return out
