"""GPU parity on randomly drawn configurations (same bars as test_gpu_parity.py): layer counts and
sizes around the tile, chunk and vector boundaries, mixed value recipes per layer (ties, zeros,
denormal and huge scales, g = h), arbitrary ratio grids, budgets from starved to unbounded, exact and
discretised cost axes, both profiles, with and without reuse of the profile's thresholds."""
import numpy as np
import pytest

from kimad_synth.gen import Workload, paper_grid
from tests.test_gpu_parity import _full_check

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 5, 63, 64, 65, 255, 1000, 1023, 1025, 4096, 5000, 16385, 70001, 200003, 1000003]
SIZE_P = np.array([2, 1, 1, 1, 1, 1, 1, 2, 1, 1, 2, 2, 2, 3, 2, 1], dtype=np.float64)


def _layer(rng, n):
    kind = rng.choice(["normal", "t", "laplace", "quantised", "sparse", "constant", "tiny", "huge", "mixed"])
    scale = 10.0 ** rng.uniform(-4, 1)
    if kind == "normal":
        v = rng.standard_normal(n) * scale
    elif kind == "t":
        v = rng.standard_t(2.5, n) * scale
    elif kind == "laplace":
        v = rng.laplace(0.0, scale, n)
    elif kind == "quantised":
        v = np.round(rng.standard_normal(n) * 4.0) / 4.0 * scale
    elif kind == "sparse":
        v = rng.standard_normal(n) * scale * (rng.random(n) < 0.1)
    elif kind == "constant":
        v = np.where(rng.random(n) < 0.5, -scale, scale) * np.ones(n)
    elif kind == "tiny":
        v = rng.standard_normal(n) * 1e-41
    elif kind == "huge":
        v = rng.standard_normal(n) * 1e17
    else:
        v = rng.standard_normal(n) * 10.0 ** rng.uniform(-8, 2, size=n)
    return v.astype(np.float32), kind


def random_workload(seed):
    rng = np.random.default_rng([2312, 8053, seed])
    L = int(rng.integers(1, 11))
    sizes = rng.choice(SIZES, size=L, p=SIZE_P / SIZE_P.sum())
    gs, hs, kinds = [], [], []
    for n in sizes.tolist():
        g, kind = _layer(rng, n)
        hk = rng.choice(["zero", "half", "same"], p=[0.5, 0.4, 0.1])
        if hk == "zero":
            h = np.zeros(n, np.float32)
        elif hk == "half":
            h = (0.5 * _layer(rng, n)[0]).astype(np.float32)
        else:
            h = g.copy()
        gs.append(g); hs.append(h); kinds.append(kind + "/" + hk)
    gk = rng.choice(["log", "uniform", "paper", "single"])
    if gk == "log":
        J = int(rng.integers(2, 65))
        ratios = np.unique(np.logspace(rng.uniform(-6, -2), 0.0 if rng.random() < 0.6 else rng.uniform(-2, 0), J))
    elif gk == "uniform":
        ratios = np.unique(rng.uniform(1e-4, 1.0, int(rng.integers(1, 40))))
    elif gk == "paper":
        ratios = paper_grid()
    else:
        ratios = np.array([rng.choice([1e-3, 0.05, 0.5, 1.0])])
    ratios = ratios[(ratios > 0) & (ratios <= 1.0)]
    d = int(sizes.sum())
    frac = float(rng.choice([0.0005, 0.01, 0.1, 0.5, 1.5]))
    D = int(rng.choice([0, 0, 3, 50, 1000, 5000]))
    budget = int(frac * 4 * d)
    # the exact cost axis has one cell per pair: keep it within the plan's row storage for the test
    if D == 0 and budget // 8 > 400000:
        D = 1000
    w = Workload(name=f"random{seed}", sizes=sizes.astype(np.uint64), g=np.concatenate(gs), h=np.concatenate(hs),
                 ratios=ratios.astype(np.float64), budget_bytes=budget, cost_units_D=D,
                 meta={"kinds": kinds, "grid": gk})
    opts = dict(reuse=bool(rng.random() < 0.6), classic=bool(rng.random() < 0.25), hint=bool(rng.random() < 0.7))
    return w, opts


# (seeds 102 to 563: configurations of small layers only, with the two-pass profile and reuse of its thresholds)
@pytest.mark.parametrize("seed", list(range(24)) + [102, 161, 249, 331, 523, 563])
def test_random_configuration(seed):
    w, opts = random_workload(seed)
    print(seed, w.sizes.tolist(), w.meta, len(w.ratios), w.budget_bytes, w.cost_units_D, opts, flush=True)
    _full_check(w, **opts)
