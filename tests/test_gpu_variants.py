"""GPU parity of the variants: dense fallback of the allocation (Section 4.2's levelling off at the uncompressed
size) and half-precision payload values (Section 2.2), both against the oracle, bit for bit."""
import numpy as np
import pytest

import kimad_synth as ks
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu

DENSE = 8


@pytest.mark.parametrize("dp", [2, 4])                     # whole rows / band
@pytest.mark.parametrize("frac,D", [(0.3, 1000), (0.6, 300), (0.05, 0), (2.0, 1000)])
def test_dense_fallback_allocation_and_compression(frac, D, dp):
    import torch
    import paper_2312_08053_amd as kimad
    work = ks.make_workload("gpt2", n_layer=1, vocab=2053, budget_frac=frac / 4 * 4, D=D)
    budget = int(frac * 4 * work.d)
    g, h = gh.to_device(work)
    sizes = work.sizes.tolist()
    plan = kimad.Plan(g, h, sizes, work.ratios.tolist(), D=D, max_budget_bytes=max(budget, 8), cfg_flags=DENSE | dp)
    gL, hL = gh.oracle_layers(work)
    E_ref, Kt = ko.profile(gL, hL, work.ratios)
    E_gpu = plan.profile(budget_hint_bytes=budget).cpu().numpy().reshape(work.L, -1)
    gh.assert_table_close(E_gpu, E_ref, Kt, work.sizes)
    st, j_ref, K_ref, off_ref = ko.allocate(E_gpu, Kt, budget, 8, D, dense_sizes=sizes)
    j, K, off, status = plan.allocate(budget)
    torch.cuda.synchronize()
    assert int(status.item()) == st == 0
    assert np.array_equal(j.cpu().numpy(), j_ref)
    assert np.array_equal(K.cpu().numpy().astype(np.uint64), K_ref)
    assert np.array_equal(off.cpu().numpy().astype(np.uint64), off_ref)
    # what is charged stays within the budget although more pairs than budget / 8 may be sent
    Ev, Kc, Ks = ko.dense_view(E_gpu, Kt, sizes, 8)
    assert 8 * sum(int(Kc[i, j_ref[i]]) for i in range(work.L)) <= budget
    if frac >= 0.3:
        assert any(int(K_ref[i]) == sizes[i] and Kt[i, j_ref[i]] < sizes[i] for i in range(work.L)), "no layer went dense"
    if frac >= 2.0:
        assert list(K_ref) == sizes                        # the plateau: everything, error 0
    idx, val, cstat = plan.compress_ef(reuse_profile=True)
    torch.cuda.synchronize()
    assert int(cstat.item()) == 0
    gh.check_compress(work, plan, h, K_ref, off_ref, idx, val)


@pytest.mark.parametrize("name,kw", [("mlp", {}), ("gpt2", dict(n_layer=1, vocab=2053, h_factor=0.5))])
def test_half_precision_values_worker_and_server(name, kw):
    import torch
    import paper_2312_08053_amd as kimad
    work = ks.make_workload(name, **kw)
    # values around and beyond the ends of the binary16 range: saturation and underflow must match too
    scale = np.ones(work.d, np.float32)
    scale[::97] = 1e7
    scale[5::89] = 1e-6
    work.g = (work.g * scale).astype(np.float32)
    g, h = gh.to_device(work)
    plan = kimad.Plan(g, h, work.sizes.tolist(), work.ratios.tolist(), D=work.cost_units_D,
                      max_budget_bytes=work.budget_bytes, value_format=1)
    assert plan.pair_bytes == 6 and plan.val.dtype == torch.float16
    status = plan.step(work.budget_bytes)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    gL, hL = gh.oracle_layers(work)
    E_gpu = plan.err_table.cpu().numpy().reshape(work.L, -1)
    Kt = plan.grid_sizes()
    st, j_ref, K_ref, off_ref = ko.allocate(E_gpu, Kt, work.budget_bytes, 6, work.cost_units_D)
    assert st == 0 and np.array_equal(plan.K.cpu().numpy().astype(np.uint64), K_ref)
    assert 6 * int(off_ref[-1]) <= work.budget_bytes
    idx = gh.u32(plan.idx)
    bits = plan.val.cpu().numpy().view(np.uint16)
    h_new = h.cpu().numpy()
    saw_saturated = saw_flushed = False
    for i in range(work.L):
        li, lb, lh = ko.compress_ef_layer(gL[i], hL[i], int(K_ref[i]), value_format="f16")
        a, b = int(off_ref[i]), int(off_ref[i + 1])
        assert np.array_equal(idx[a:b], li), i
        assert np.array_equal(bits[a:b], lb), i
        assert np.array_equal(h_new[work.starts[i]:work.starts[i + 1]].view(np.uint32), lh.view(np.uint32)), i
        saw_saturated |= bool(np.any((lb & 0x7FFF) == 0x7BFF))
        saw_flushed |= bool(np.any((lb & 0x7FFF) == 0))
    assert saw_saturated
    # the server decodes the same payload into its copy of the estimator: equal to the worker's, bit for bit
    server = torch.from_numpy(work.h).cuda()
    starts = torch.from_numpy(np.asarray(work.starts, dtype=np.int64)).cuda()
    sstat = kimad.kimad_server_apply([(plan.idx, plan.val, plan.offsets)], [server], [1.0], starts, work.d)
    torch.cuda.synchronize()
    assert sstat.cpu().tolist() == [0]
    assert torch.equal(server.view(torch.int32), h.view(torch.int32))
