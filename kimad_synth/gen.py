"""Seeded value recipes for the synthetic gradient sets.

Every set is a flat fp32 buffer ``g`` (the fresh update), a flat fp32 buffer
``h`` (the error-feedback estimator), per-layer sizes, a ratio grid and a byte
budget.  Layers sit back to back in the flat buffers, so segment starts are
only 4-byte aligned, as they are inside a framework's flattened gradient bucket.

Draw order (fixed, so both consumers see identical bits):
    rng = numpy.random.default_rng([seed, workload_id, step])
    1. the L per-layer scales, one draw each, in layer order;
    2. ``g`` layer by layer (plus that layer's outlier mask where the recipe has one);
    3. ``h`` layer by layer (recipes with a non-zero estimator only).
Values are drawn in float64 and cast to float32 once.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from . import shapes as _shapes


@dataclass
class Workload:
    name: str
    sizes: np.ndarray            # uint64[L], elements per layer
    g: np.ndarray                # float32[d]
    h: np.ndarray                # float32[d]
    ratios: np.ndarray           # float64[J], ascending, in (0, 1]
    budget_bytes: int
    cost_units_D: int            # 0 = exact knapsack
    pair_bytes: int = 8
    meta: dict = field(default_factory=dict)

    @property
    def L(self) -> int:
        return int(self.sizes.shape[0])

    @property
    def d(self) -> int:
        return int(self.sizes.sum())

    @property
    def starts(self) -> np.ndarray:
        s = np.zeros(self.L + 1, dtype=np.int64)
        np.cumsum(self.sizes.astype(np.int64), out=s[1:])
        return s

    def layer_views(self, arr: np.ndarray) -> List[np.ndarray]:
        s = self.starts
        return [arr[s[i]:s[i + 1]] for i in range(self.L)]


def ratio_grid(lo_exp: float, hi_exp: float, J: int) -> np.ndarray:
    """J log-spaced ratios 10**lo_exp .. 10**hi_exp (hi_exp = 0 ends at exactly 1.0)."""
    r = np.logspace(lo_exp, hi_exp, J, dtype=np.float64)
    r[-1] = 10.0 ** hi_exp
    return r


def paper_grid() -> np.ndarray:
    """The grid of Section 4.3: {0.01 + 0.02 k <= 1}, 50 values."""
    return np.array([0.01 + 0.02 * k for k in range(50)], dtype=np.float64)


def _sizes(shape_list: Sequence[Sequence[int]]) -> np.ndarray:
    return np.array([_shapes.numel(s) for s in shape_list], dtype=np.uint64)


def _log_uniform(rng: np.random.Generator, lo: float, hi: float, L: int) -> np.ndarray:
    return 10.0 ** rng.uniform(lo, hi, size=L)


def _fill(sizes: np.ndarray, draw: Callable[[int, int], np.ndarray]) -> np.ndarray:
    d = int(sizes.sum())
    out = np.empty(d, dtype=np.float32)
    pos = 0
    for i, n in enumerate(sizes.tolist()):
        out[pos:pos + n] = draw(i, n)
        pos += n
    return out


def _make(name: str, wid: int, shape_list, seed: int, step: int, dist: str, scale_range,
          h_factor: float, ratios: np.ndarray, budget_frac: float, D: int,
          outlier_p: float = 0.0, outlier_mult: float = 1.0,
          scale_rng_step: Optional[int] = None, scales_of_step: Optional[int] = None) -> Workload:
    sizes = _sizes(shape_list)
    L = len(sizes)
    # Scales may be tied to a fixed step so that they persist across a multi-step chain.
    if scales_of_step is not None:
        # another round of the same model: the per-layer scales of the set drawn for step `scales_of_step` (its
        # first L draws), fresh values from a stream of their own
        scale = _log_uniform(np.random.default_rng([seed, wid, scales_of_step]), scale_range[0], scale_range[1], L)
        rng = np.random.default_rng([seed, wid, step, 1])
    elif scale_rng_step is None:
        rng = np.random.default_rng([seed, wid, step])
        scale = _log_uniform(rng, scale_range[0], scale_range[1], L)
    else:
        scale = _log_uniform(np.random.default_rng([seed, wid, scale_rng_step, 7]),
                             scale_range[0], scale_range[1], L)
        rng = np.random.default_rng([seed, wid, step])

    def base(n: int) -> np.ndarray:
        if dist == "normal":
            return rng.standard_normal(n)
        if dist == "laplace":
            return rng.laplace(0.0, 1.0, n)
        if dist.startswith("t"):
            return rng.standard_t(float(dist[1:]), n)
        raise ValueError(dist)

    def draw_g(i: int, n: int) -> np.ndarray:
        v = base(n) * scale[i]
        if outlier_p > 0.0:
            mask = rng.random(n) < outlier_p
            v[mask] *= outlier_mult
        return v

    g = _fill(sizes, draw_g)
    if h_factor != 0.0:
        h = _fill(sizes, lambda i, n: base(n) * (h_factor * scale[i]))
    else:
        h = np.zeros(int(sizes.sum()), dtype=np.float32)
    d = int(sizes.sum())
    budget = int(np.floor(budget_frac * 4 * d))
    return Workload(name=name, sizes=sizes, g=g, h=h, ratios=ratios, budget_bytes=budget,
                    cost_units_D=D, meta={"seed": seed, "step": step, "dist": dist})


def make_workload(name: str, seed: int = 0, step: int = 0, **kw) -> Workload:
    """Build one of the named synthetic sets.

    ``mlp``        6 tensors, N(0, s^2), s = 10^U(-4,-1), h = 0, 16 ratios 1e-3..1, budget 10 %.
    ``resnet18``   62 tensors, s * t(3), s = 10^U(-5,-2), h = 0.5 s * t(3), 32 ratios 1e-4..1, budget 1 %.
    ``resnet50``   161 tensors, Laplace(0, b), b = 10^U(-6,-2), h = 0, 32 ratios, budget_frac in {0.001, 0.01, 0.05}.
    ``gpt2``       148 tensors, s * t(2.5), 0.1 % of entries x100, h = 0 (or ``h_factor=0.5``), 64 ratios 1e-5..1, budget 1 %.
    ``llama``      218 tensors, s * t(3) with per-layer scales fixed across steps, h = 0, 64 ratios 1e-5..1.
    Keyword overrides: ``budget_frac``, ``D``, ``h_factor``, and the shape arguments of the
    architecture (``n_layer``, ``vocab`` ...) to build reduced variants of the same recipe.
    """
    budget_frac = kw.pop("budget_frac", None)
    D = kw.pop("D", None)
    h_factor = kw.pop("h_factor", None)
    scales_of_step = kw.pop("scales_of_step", None)       # gpt2 only: a later round with the scales of an earlier set
    if name == "mlp":
        return _make("mlp", 1, _shapes.mlp_shapes(), seed, step, "normal", (-4, -1),
                     0.0 if h_factor is None else h_factor, ratio_grid(-3, 0, 16),
                     0.10 if budget_frac is None else budget_frac, 0 if D is None else D)
    if name == "resnet18":
        return _make("resnet18", 2, _shapes.resnet18_shapes(**kw), seed, step, "t3", (-5, -2),
                     0.5 if h_factor is None else h_factor, ratio_grid(-4, 0, 32),
                     0.01 if budget_frac is None else budget_frac, 0 if D is None else D)
    if name == "resnet50":
        return _make("resnet50", 3, _shapes.resnet50_shapes(**kw), seed, step, "laplace", (-6, -2),
                     0.0 if h_factor is None else h_factor, ratio_grid(-4, 0, 32),
                     0.01 if budget_frac is None else budget_frac, 0 if D is None else D)
    if name == "gpt2":
        return _make("gpt2", 4, _shapes.gpt2_small_shapes(**kw), seed, step, "t2.5", (-5, -2),
                     0.0 if h_factor is None else h_factor, ratio_grid(-5, 0, 64),
                     0.01 if budget_frac is None else budget_frac, 1000 if D is None else D,
                     outlier_p=1e-3, outlier_mult=100.0, scales_of_step=scales_of_step)
    if name == "llama":
        return _make("llama", 5, _shapes.llama_shapes(**kw), seed, step, "t3", (-5, -2),
                     0.0 if h_factor is None else h_factor, ratio_grid(-5, 0, 64),
                     0.01 if budget_frac is None else budget_frac, 1000 if D is None else D,
                     scale_rng_step=0)
    raise KeyError(name)


WORKLOADS: Dict[str, dict] = {
    "mlp": dict(L=6, d=235_146),
    "resnet18": dict(L=62, d=11_689_512),
    "resnet50": dict(L=161, d=25_557_032),
    "gpt2": dict(L=148, d=124_439_808),
    "llama": dict(L=218, d=1_298_761_728),
}


def bandwidth_trace(steps: int, seed: int = 0, b0: float = 5.5, sigma: float = 0.5,
                    lo: float = 1.0, hi: float = 10.0) -> np.ndarray:
    """Seeded random-walk bandwidth in Gbit/s, reflected into [lo, hi]."""
    rng = np.random.default_rng([seed, 5, 1_000_003])
    out = np.empty(steps, dtype=np.float64)
    b = b0
    for k in range(steps):
        out[k] = b
        b = b + rng.normal(0.0, sigma)
        while b < lo or b > hi:
            if b < lo:
                b = 2 * lo - b
            if b > hi:
                b = 2 * hi - b
    return out


def sin2_bandwidth_trace(times: Sequence[float], eta: float = 300e6, theta: float = 0.05,
                         delta: float = 30e6, noise: float = 0.0, seed: int = 0) -> np.ndarray:
    """The bandwidth pattern of the paper's deep-model experiment (Section 4.2, Bandwidth):
    eta * sin(theta * time)^2 + delta in bits per second; the defaults span its 30..330 Mbps.
    `noise` adds seeded Gaussian noise of that relative size per worker, clipped at delta / 2."""
    t = np.asarray(times, dtype=np.float64)
    b = eta * np.sin(theta * t) ** 2 + delta
    if noise > 0.0:
        rng = np.random.default_rng([seed, 5, 2_000_003])
        b = np.maximum(b * (1.0 + noise * rng.standard_normal(b.shape)), delta / 2.0)
    return b


def budget_from_bandwidth(gbit_per_s: float, seconds: float = 0.05) -> int:
    """Bytes that fit through a link of the given rate in the given time."""
    return int(np.floor(gbit_per_s * 1e9 * seconds / 8.0))
