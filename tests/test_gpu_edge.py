"""GPU parity on adversarial and degenerate inputs (same bars as test_gpu_parity.py)."""
import numpy as np
import pytest

import kimad_synth as ks
from kimad_synth.gen import Workload, paper_grid
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh
from tests.test_gpu_parity import _full_check

pytestmark = pytest.mark.gpu


def _work(layers_g, layers_h, ratios, budget_frac=0.25, D=0, name="edge"):
    sizes = np.array([len(x) for x in layers_g], dtype=np.uint64)
    g = np.concatenate(layers_g).astype(np.float32)
    h = np.concatenate(layers_h).astype(np.float32)
    budget = int(budget_frac * 4 * int(sizes.sum()))
    return Workload(name=name, sizes=sizes, g=g, h=h, ratios=np.asarray(ratios, dtype=np.float64),
                    budget_bytes=budget, cost_units_D=D)


GRID = np.array([1e-4, 1e-3, 0.01, 0.05, 0.1, 0.25, 0.5, 0.75, 0.9, 0.999, 1.0])


def test_all_equal_magnitudes():
    n_big, n_small = 20011, 777
    big = np.full(n_big, 0.5, np.float32)
    big[::2] *= -1
    small = np.full(n_small, -3.0, np.float32)
    w = _work([big, small], [np.zeros(n_big, np.float32), np.zeros(n_small, np.float32)], GRID)
    _full_check(w)
    _full_check(w, reuse=False)


def test_signed_zeros_and_few_nonzeros():
    rng = np.random.default_rng(1)
    n = 30000
    x = np.zeros(n, np.float32)
    x[1::2] = -0.0
    nz = rng.choice(n, 50, replace=False)
    x[nz] = rng.standard_normal(50).astype(np.float32)
    w = _work([x, x[:5000].copy()], [np.zeros(n, np.float32), np.zeros(5000, np.float32)], GRID, budget_frac=0.6)
    _full_check(w)


def test_denormals_only():
    rng = np.random.default_rng(2)
    n = 25000
    bits = rng.integers(0, 1 << 23, size=n, dtype=np.uint32)        # exponent field 0
    bits[::3] |= np.uint32(0x80000000)
    x = bits.view(np.float32)
    tiny = rng.integers(0, 1 << 10, size=9000, dtype=np.uint32).view(np.float32)   # below 2^-139
    w = _work([x, tiny.copy(), x[:4000].copy()],
              [np.zeros(n, np.float32), np.zeros(9000, np.float32), np.zeros(4000, np.float32)], GRID)
    _full_check(w)


def test_denormal_differences_are_kept():
    # x = g - h lands in the denormal range although g and h are normal
    rng = np.random.default_rng(3)
    n = 12000
    h = (rng.standard_normal(n) * 1e-37).astype(np.float32)
    delta = (rng.integers(-200, 200, size=n).astype(np.float64) * 1.4e-45)
    g = (h.astype(np.float64) + delta).astype(np.float32)
    w = _work([g], [h], GRID)
    x = g - h
    assert np.any((np.abs(x) > 0) & (np.abs(x) < 1.2e-38))
    _full_check(w)


def test_single_huge_outlier():
    rng = np.random.default_rng(4)
    n = 50000
    x = (rng.standard_normal(n) * 1e-6).astype(np.float32)
    x[31337] = 3e30
    s = (rng.standard_normal(100) * 1e-6).astype(np.float32)
    s[7] = -1e25
    w = _work([x, s], [np.zeros(n, np.float32), np.zeros(100, np.float32)], GRID, budget_frac=0.01)
    _full_check(w)


def test_layer_sizes_and_unaligned_segments():
    rng = np.random.default_rng(5)
    sizes = [1, 2, 63, 64, 65, 1023, 8192, 8193, 16385, 40001, 3, 9000]
    g = [rng.standard_t(3, n).astype(np.float32) * 10.0 ** rng.uniform(-4, 0) for n in sizes]
    h = [(0.5 * rng.standard_t(3, n)).astype(np.float32) * 1e-2 for n in sizes]
    w = _work(g, h, GRID, budget_frac=0.1)
    _full_check(w)
    _full_check(w, reuse=False)


def test_g_and_h_with_different_alignment():
    import torch
    import paper_2312_08053_amd as kimad
    rng = np.random.default_rng(6)
    sizes = [10007, 20000, 555]
    work = _work([rng.standard_normal(n).astype(np.float32) for n in sizes],
                 [rng.standard_normal(n).astype(np.float32) * 0.2 for n in sizes], GRID, budget_frac=0.2)
    gbuf = torch.zeros(work.d + 8, dtype=torch.float32, device="cuda")
    hbuf = torch.zeros(work.d + 8, dtype=torch.float32, device="cuda")
    g = gbuf[1:1 + work.d]
    h = hbuf[3:3 + work.d]
    g.copy_(torch.from_numpy(work.g))
    h.copy_(torch.from_numpy(work.h))
    starts = work.starts
    gl = [g[starts[i]:starts[i + 1]] for i in range(work.L)]
    hl = [h[starts[i]:starts[i + 1]] for i in range(work.L)]
    plan = kimad.Plan(gl, hl, work.sizes.tolist(), work.ratios.tolist(), max_budget_bytes=work.budget_bytes)
    plan.step(work.budget_bytes)
    torch.cuda.synchronize()
    assert plan.status.cpu().tolist() == [0, 0]
    gL, hL = gh.oracle_layers(work)
    E_ref, Kt = ko.profile(gL, hL, work.ratios)
    gh.assert_table_close(plan.err_table.cpu().numpy(), E_ref, Kt, work.sizes)
    st, j, K, off = ko.allocate(plan.err_table.cpu().numpy().reshape(work.L, -1), Kt, work.budget_bytes, 8, 0)
    assert st == 0 and np.array_equal(plan.K.cpu().numpy().astype(np.uint64), K)
    gh.check_compress(work, plan, h, K, off, plan.idx, plan.val)
    assert float(hbuf[:3].abs().sum()) == 0.0 and float(hbuf[3 + work.d:].abs().sum()) == 0.0


def test_heavily_quantised_values_many_ties_at_the_threshold():
    rng = np.random.default_rng(7)
    n = 70000
    x = (rng.integers(-12, 13, size=n) / 8.0).astype(np.float32)     # 25 distinct values
    s = (rng.integers(-3, 4, size=3000)).astype(np.float32)
    w = _work([x, s], [np.zeros(n, np.float32), np.zeros(3000, np.float32)], GRID, budget_frac=0.3)
    _full_check(w)
    _full_check(w, reuse=False)


def test_paper_grid_and_discretisation_factor():
    rng = np.random.default_rng(8)
    sizes = [30000, 512, 9000, 100000, 64]
    g = [rng.laplace(0, 1, n).astype(np.float32) * 10.0 ** rng.uniform(-5, -1) for n in sizes]
    h = [np.zeros(n, np.float32) for n in sizes]
    _full_check(_work(g, h, paper_grid(), budget_frac=0.08, D=1000))


def test_nonfinite_entries_are_ranked_first_and_reported():
    import torch
    rng = np.random.default_rng(9)
    n = 20000
    x = rng.standard_normal(n).astype(np.float32)
    x[5] = np.inf
    x[17] = -np.inf
    x[[4000, 4001, 9000]] = np.nan
    s = rng.standard_normal(300).astype(np.float32)
    s[3] = np.nan
    work = _work([x, s], [np.zeros(n, np.float32), np.zeros(300, np.float32)],
                 [1e-4, 1.5e-4, 0.01, 0.5, 1.0], budget_frac=0.2)
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    gL, hL = gh.oracle_layers(work)
    E_ref, Kt = ko.profile(gL, hL, work.ratios)
    E = plan.profile().cpu().numpy().reshape(work.L, -1)
    assert np.isnan(E_ref[0, 0]) and np.isinf(E_ref[0, 1]) and np.isfinite(E_ref[0, 2])   # K = 2, 3, 200
    gh.assert_table_close(E, E_ref, Kt, work.sizes)
    j, K, off, st = plan.allocate(work.budget_bytes)
    assert int(st.item()) == ko.ERR_NONFINITE and int(off.cpu().numpy().sum()) == 0
    # selection itself is well defined: NaN patterns rank above Inf, Inf above everything else
    K_ref = np.array([3, 1], dtype=np.uint64)
    off_ref = np.array([0, 3, 4], dtype=np.uint64)
    idx, val, cst = plan.compress_ef(torch.from_numpy(K_ref.astype(np.int64)).cuda(),
                                     torch.from_numpy(off_ref.astype(np.int64)).cuda(), reuse_profile=False)
    assert int(cst.item()) == 0
    assert gh.u32(idx)[:4].tolist() == [4000, 4001, 9000, 3]


def test_zero_and_full_k_and_infeasible_budget():
    import torch
    work = ks.make_workload("mlp")
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    sizes = work.sizes.astype(np.int64)
    K_ref = np.array([0, sizes[1], sizes[2], 0, 7, sizes[5]], dtype=np.uint64)
    off_ref = np.concatenate([[0], np.cumsum(K_ref)]).astype(np.uint64)
    idx, val, cst = plan.compress_ef(torch.from_numpy(K_ref.astype(np.int64)).cuda(),
                                     torch.from_numpy(off_ref.astype(np.int64)).cuda(), reuse_profile=False)
    assert int(cst.item()) == 0
    gh.check_compress(work, plan, h, K_ref, off_ref, idx, val)
    plan.profile()
    _, _, _, st = plan.allocate(8 * (work.L - 1))
    assert int(st.item()) == ko.ERR_INFEASIBLE


def test_device_side_refusals_leave_h_untouched():
    import torch
    import paper_2312_08053_amd as kimad
    work = ks.make_workload("mlp")
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    plan.profile()
    Kt = plan.grid_sizes()
    K = torch.from_numpy(Kt[:, 3].copy()).cuda()
    off = torch.zeros(work.L + 1, dtype=torch.int64, device="cuda")
    off[1:] = torch.cumsum(K, 0)
    bad = K.clone()
    bad[0] += 1                                           # not a grid size
    _, _, st = plan.compress_ef(bad, off, reuse_profile=True)
    assert int(st.item()) == -8
    off_bad = off.clone()
    off_bad[2] = plan.capacity_pairs                      # would run past the payload buffers
    _, _, st = plan.compress_ef(K, off_bad, reuse_profile=True)
    assert int(st.item()) == -10
    assert np.array_equal(h.cpu().numpy().view(np.uint32), work.h.view(np.uint32))
    _, _, st = plan.compress_ef(K, off, reuse_profile=True)
    assert int(st.item()) == 0
    gh.check_compress(work, plan, h, Kt[:, 3], off.cpu().numpy(), plan.idx, plan.val)
    # The compression changed h: the profile's thresholds no longer describe g - h.  A retry that reuses them
    # (say after a failed send) is refused and changes nothing; Section 3.3's estimator equality would break otherwise.
    h_after = h.cpu().numpy().copy()
    plan.idx.zero_()
    _, _, st = plan.compress_ef(K, off, reuse_profile=True)
    torch.cuda.synchronize()
    assert int(st.item()) == -12
    assert np.array_equal(h.cpu().numpy().view(np.uint32), h_after.view(np.uint32))
    assert not plan.idx.cpu().numpy().any()
    # a selection from scratch needs no profile; it too ends the validity of an earlier one
    plan.profile()
    _, _, st = plan.compress_ef(K, off, reuse_profile=False)
    assert int(st.item()) == 0
    _, _, st = plan.compress_ef(K, off, reuse_profile=True)
    assert int(st.item()) == -12
    # and a plan that has never been profiled refuses the reuse as well
    plan2 = gh.make_plan(work, g, h)
    _, _, st = plan2.compress_ef(K, off, reuse_profile=True)
    assert int(st.item()) == -12


def test_allocate_refuses_a_budget_beyond_the_plans_tables():
    import paper_2312_08053_amd as kimad
    work = ks.make_workload("mlp")                        # exact cost axis: the tables hold max_budget_bytes / 8 cells
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h, max_budget_bytes=8 * 1000)
    plan.profile()
    with pytest.raises(kimad.KimadError) as e:
        plan.allocate(8 * 5000)
    assert e.value.code == -1
    plan.allocate(8 * 1000)
    assert int(plan.status[0].item()) == 0


def _hash32(a):
    a &= 0xFFFFFFFF
    a ^= a >> 16; a = (a * 0x7feb352d) & 0xFFFFFFFF
    a ^= a >> 15; a = (a * 0x846ca68b) & 0xFFFFFFFF
    a ^= a >> 16
    return a


def test_sample_that_misleads_the_prediction_is_recounted():
    # The single-pass profile reads one 1024-entry chunk in every `stride` first.  Make exactly those
    # chunks huge and the rest ordinary: the bins predicted for the dense candidates are all wrong,
    # and the layer must be recounted by the full pass with the same exact results.
    rng = np.random.default_rng(10)
    n = 1024 * 1024
    nchunks = n // 1024
    stride = max(1, min(16, nchunks // 64))
    x = rng.standard_normal(n).astype(np.float32)
    for grp in range((nchunks + stride - 1) // stride):
        c = grp * stride + _hash32((grp * 2654435761 + 12345) & 0xFFFFFFFF) % stride
        if c < nchunks:
            x[c * 1024:(c + 1) * 1024] *= 1e6
    # 16-byte aligned start, so that chunks of the layer are chunks of the buffer
    w = _work([x], [np.zeros(n, np.float32)], GRID, budget_frac=0.02)
    _full_check(w, expect_redo=1)


def test_results_are_reproducible_and_profile_is_pure():
    """The table is a function of g, h and the grid alone: whatever an earlier call on other data left in the
    plan's workspace (candidates, histograms, the history the next prediction starts from, allocation rows), the
    same input gives the same bits.  Between two profiles of one input the plan runs a whole step on an unrelated
    one (every layer scaled differently, values permuted)."""
    import torch
    work = ks.make_workload("resnet18")
    g, h = gh.to_device(work)
    g0, h0 = g.clone(), h.clone()
    plan = gh.make_plan(work, g, h)
    a = plan.profile().clone()
    other = ks.make_workload("resnet18", step=3)
    g.copy_(torch.from_numpy(other.g * np.float32(37.0)).flip(0))
    st = plan.step(work.budget_bytes)
    torch.cuda.synchronize()
    assert st.cpu().tolist() == [0, 0]
    g.copy_(g0); h.copy_(h0)
    b = plan.profile().clone()
    plan2 = gh.make_plan(work, g, h)
    fresh = plan2.profile().clone()
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int64), b.view(torch.int64)), "table must be bit-reproducible"
    assert torch.equal(a.view(torch.int64), fresh.view(torch.int64)), "and the same on a new plan"


@pytest.mark.parametrize("classic", [False, True])
def test_profile_of_small_layers_only_can_be_reused(classic):
    """A plan without a tiled layer: the small layers' kernel, on the side stream, is the only one that marks the
    profile as fresh, and the clearing at the start of a profile must not overtake it (it did in the two-pass
    profile: the compression then refused to reuse the thresholds, status STALE_PROFILE)."""
    rng = np.random.default_rng(161)
    sizes = [63, 1023, 4096, 5000, 1]
    gs = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    hs = [np.zeros(n, np.float32) for n in sizes]
    hs[1] = (0.5 * rng.standard_normal(1023)).astype(np.float32)
    w = _work(gs, hs, GRID, budget_frac=0.1, D=50)
    for _ in range(3):                                    # the race did not lose every time
        _full_check(w, reuse=True, classic=classic)
