"""kimad_allocate_static, the allocation for callers that cannot allocate: same outputs as
kimad_allocate, bit for bit, on two calls in a row that share the library's fixed tables, the second
on a smaller problem (fewer layers, a smaller budget, shorter rows)."""
import numpy as np
import pytest

import kimad_synth as ks
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _both(work, budget):
    import torch
    import paper_2312_08053_amd as kimad
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    plan.profile(budget_hint_bytes=budget)
    dev = g.device
    # poison the outputs of the new entry point so that a call that writes nothing cannot pass
    j = torch.full((work.L,), -7, dtype=torch.int32, device=dev)
    K = torch.full((work.L,), -7, dtype=torch.int64, device=dev)
    off = torch.full((work.L + 1,), -7, dtype=torch.int64, device=dev)
    st = torch.full((1,), -99, dtype=torch.int32, device=dev)
    kimad.kimad_allocate_static(plan.handle, plan.err_table, budget, j, K, off, st)
    torch.cuda.synchronize()
    got = (j.cpu().numpy().copy(), K.cpu().numpy().copy(), off.cpu().numpy().copy(), int(st.item()))
    j2, K2, off2, st2 = plan.allocate(budget)
    torch.cuda.synchronize()
    want = (j2.cpu().numpy(), K2.cpu().numpy(), off2.cpu().numpy(), int(st2.item()))
    assert got[3] == want[3]
    for a, b, name in zip(got[:3], want[:3], ("j", "K", "offsets")):
        assert np.array_equal(a, b), name
    return got


def test_static_tables_give_the_same_allocation_twice_in_a_row():
    big = ks.make_workload("resnet50", D=1000)                       # 161 layers, rows of about 1000 cells
    j1, K1, off1, st1 = _both(big, big.budget_bytes)
    assert st1 == 0 and int(off1[-1]) * 8 <= big.budget_bytes and K1.min() >= 1
    small = ks.make_workload("mlp", D=200)                           # 6 layers, rows of about 200 cells
    j2, K2, off2, st2 = _both(small, small.budget_bytes // 3)
    assert st2 == 0 and int(off2[-1]) * 8 <= small.budget_bytes // 3
    # an infeasible budget is reported the same way, and leaves the outputs zero-filled
    j3, K3, off3, st3 = _both(small, 8)
    assert st3 == -6 and not K3.any() and not off3.any()


def test_static_tables_refuse_what_they_cannot_hold():
    import torch
    import paper_2312_08053_amd as kimad
    work = ks.make_workload("resnet18", D=3000)                      # rows of about 3000 cells: beyond the fixed tables
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    plan.profile()
    j, K, off, st = plan.j, plan.K, plan.offsets, plan.status[0:1]
    with pytest.raises(kimad.KimadError) as e:
        kimad.kimad_allocate_static(plan.handle, plan.err_table, work.budget_bytes, j, K, off, st)
    assert e.value.code == -11
    # too many layers
    sizes = [64] * 300
    n = sum(sizes)
    g2 = torch.randn(n, device="cuda")
    h2 = torch.zeros(n, device="cuda")
    p2 = kimad.Plan(g2, h2, sizes, [0.1, 0.5, 1.0], D=100, max_budget_bytes=8 * n)
    p2.profile()
    with pytest.raises(kimad.KimadError) as e:
        kimad.kimad_allocate_static(p2.handle, p2.err_table, 8 * n // 4, p2.j, p2.K, p2.offsets, p2.status[0:1])
    assert e.value.code == -11
