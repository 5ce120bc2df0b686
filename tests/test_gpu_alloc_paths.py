"""kimad_allocate on tables given directly (any table is a valid input): the recurrence over whole rows and the
one inside the band that Lagrangian bounds leave must both return the oracle's dynamic programme (Appendix C)
bit for bit: the chosen j per layer, K, the offsets and the status.  The tables here are drawn to stress what the
band's construction leans on: convex and non-convex rows, runs of equal costs and equal errors, ties between
totals, one layer, one ratio, ample and starved budgets, non-finite entries, more layers than its multiplier
table of 32 holds, more list records than its LDS holds."""
import numpy as np
import pytest

from oracle import kimad_oracle as ko

pytestmark = pytest.mark.gpu

FULL, BAND = 2, 4


def _plan(sizes, ratios, D, max_budget, flags):
    import torch
    import paper_2312_08053_amd as kimad
    n = int(sum(sizes))
    g = torch.zeros(n, dtype=torch.float32, device="cuda")
    h = torch.zeros(n, dtype=torch.float32, device="cuda")
    return kimad.Plan(g, h, list(sizes), list(ratios), D=D, max_budget_bytes=max_budget, cfg_flags=flags, capacity_pairs=1)


def _check(sizes, ratios, E, budget, D, expect_band=None):
    import torch
    Kt = np.array([ko.grid_sizes(ratios, int(n)) for n in sizes])
    st_ref, j_ref, K_ref, off_ref = ko.allocate(E, Kt, budget, 8, D)
    E_dev = torch.from_numpy(np.ascontiguousarray(E, dtype=np.float64).reshape(-1)).cuda()
    infos = {}
    for flags in (FULL, BAND):
        plan = _plan(sizes, ratios, D, max(budget, 8), flags)
        assert np.array_equal(plan.grid_sizes(), Kt)
        j, K, off, st = plan.allocate(budget, E_dev)
        torch.cuda.synchronize()
        assert int(st.item()) == st_ref, (flags, int(st.item()), st_ref)
        if st_ref == ko.OK:
            assert np.array_equal(j.cpu().numpy(), j_ref), flags
            assert np.array_equal(K.cpu().numpy().astype(np.uint64), K_ref), flags
            assert np.array_equal(off.cpu().numpy().astype(np.uint64), off_ref), flags
        else:
            assert not K.cpu().numpy().any() and not off.cpu().numpy().any()
        infos[flags] = plan.allocate_diagnostics()
        plan.close()
    if expect_band is not None:
        assert infos[BAND]["whole_rows"] == (0 if expect_band else 1), infos[BAND]
    return infos[BAND]


def _convex_table(rng, sizes, ratios, scale_lo=-6, scale_hi=2):
    """Rows shaped like TopK error profiles: decreasing, convex in K, exactly 0 at K = n."""
    rows = []
    for n in sizes:
        K = ko.grid_sizes(ratios, int(n)).astype(np.float64)
        a = rng.uniform(0.3, 3.0)
        s = 10.0 ** rng.uniform(scale_lo, scale_hi)
        rows.append(s * (1.0 - K / n) ** (1.0 + a))
    return np.array(rows)


def test_profile_shaped_tables_many_budgets_and_factors():
    rng = np.random.default_rng(11)
    ratios = np.logspace(-4, 0, 40)
    for trial in range(6):
        L = int(rng.integers(2, 60))
        sizes = [int(x) for x in rng.choice([700, 5000, 70000, 300000, 2000000], size=L)]
        E = _convex_table(rng, sizes, ratios)
        d = sum(sizes)
        for frac, D in ((0.002, 1000), (0.02, 4096), (0.3, 300), (0.05, 2500)):
            info = _check(sizes, ratios, E, int(frac * 8 * d), D, expect_band=True)
            assert info["max_band"] >= 1


def test_non_convex_and_noisy_rows():
    rng = np.random.default_rng(12)
    ratios = np.linspace(0.02, 1.0, 50)
    for trial in range(6):
        L = int(rng.integers(1, 25))
        sizes = [int(x) for x in rng.integers(100, 50000, size=L)]
        E = np.sort(rng.random((L, 50)) * 10.0 ** rng.uniform(-3, 3, size=(L, 1)), axis=1)[:, ::-1].copy()
        if trial % 2:
            E = rng.random((L, 50))                      # not even monotone: a caller may pass any table
        d = sum(sizes)
        _check(sizes, ratios, E, int(rng.uniform(0.05, 0.9) * 8 * d), int(rng.choice([50, 700, 1000, 3000])))


def test_ties_equal_errors_and_equal_costs():
    rng = np.random.default_rng(13)
    ratios = np.linspace(0.1, 1.0, 10)
    sizes = [40] * 12 + [4000] * 6
    # small integers: many totals tie exactly, so the lowest j and the smallest cost must win as in the oracle
    E = np.sort(rng.integers(0, 4, size=(len(sizes), 10)).astype(np.float64), axis=1)[:, ::-1].copy()
    for D in (20, 100, 0):
        for budget in (8 * 300, 8 * 3000, 8 * 20000):
            _check(sizes, ratios, E, budget, D)
    E0 = np.zeros_like(E)
    _check(sizes, ratios, E0, 8 * 3000, 100)


def test_one_layer_one_ratio_ample_and_starved_budgets():
    ratios = np.logspace(-3, 0, 16)
    rng = np.random.default_rng(14)
    E1 = _convex_table(rng, [100000], ratios)
    _check([100000], ratios, E1, 8 * 5000, 1000)
    _check([100000], ratios, E1, 8 * 200000, 1000)                   # more than everything costs
    _check([100000], ratios, E1, 0, 1000)                            # nothing fits
    sizes = [5000, 300, 90000]
    _check(sizes, [0.25], _convex_table(rng, sizes, [0.25]), 8 * 30000, 500)
    _check(sizes, [0.25], _convex_table(rng, sizes, [0.25]), 8 * 100, 500)       # infeasible: the only ratio is too dear
    E3 = _convex_table(rng, sizes, ratios)
    d = sum(sizes)
    _check(sizes, ratios, E3, 8 * d, 1000)                           # K = n everywhere: total 0
    _check(sizes, ratios, E3, 8 * 3, 1000)                           # exactly the cheapest allocation
    _check(sizes, ratios, E3, 8 * 2, 1000)                           # one pair short of it


def test_nonfinite_tables_are_reported_by_both_paths():
    ratios = np.logspace(-2, 0, 8)
    sizes = [1000, 20000, 333]
    rng = np.random.default_rng(15)
    for bad in (np.inf, np.nan, -np.inf):
        E = _convex_table(rng, sizes, ratios)
        E[1, 3] = bad
        info = _check(sizes, ratios, E, 8 * 4000, 1000)
        assert info["whole_rows"] == 1


def test_many_layers_and_many_list_records():
    rng = np.random.default_rng(16)
    # 600 layers of 10 ratios: the multiplier table falls back to 8 columns, one thread a row
    ratios = np.logspace(-3, 0, 10)
    sizes = [int(x) for x in rng.integers(50000, 400000, size=600)]
    E = _convex_table(rng, sizes, ratios, -2, 2)
    d = sum(sizes)
    _check(sizes, ratios, E, int(0.3 * 8 * d), 4000, expect_band=True)
    # 230 layers x 64 ratios with mostly distinct costs: more list records than the bounds kernel holds in LDS,
    # so it declares whole rows and the recurrence visits every cell: same result
    ratios = np.logspace(-4, 0, 64)
    sizes = [int(x) for x in rng.integers(3000000, 4000000, size=230)]
    E = _convex_table(rng, sizes, ratios, -2, 2)
    d = sum(sizes)
    _check(sizes, ratios, E, int(0.05 * 8 * d), 4200, expect_band=False)



def test_more_layers_than_cost_cells_is_infeasible():
    """Every layer costs at least one cell: 5000 layers cannot fit rows of 601 cells, whatever the budget's size in
    bytes (the walk back, which keeps the path's cells in LDS, is never reached)."""
    rng = np.random.default_rng(23)
    ratios = [0.05, 0.3, 1.0]
    sizes = [int(x) for x in rng.integers(100, 3000, size=5000)]
    E = _convex_table(rng, sizes, ratios, -3, 1)
    d = sum(sizes)
    _check(sizes, ratios, E, int(0.25 * 8 * d), 600)
    # and with as many cells as layers allow it, through rows of 4200 cells
    sizes = sizes[:4000]
    E = E[:4000]
    _check(sizes, ratios, E, int(0.5 * 8 * sum(sizes)), 4200)
