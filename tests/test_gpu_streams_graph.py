"""One worker's step (Algorithm 1, worker lines) on a stream of the caller's, and recorded into a HIP graph.

The library enqueues everything on the stream it is given (small layers on a side stream forked from and joined
into it), waits for nothing and clears its tables with kernels, so a step can be recorded and replayed.  A replay
must give what the eager call gives, bit for bit, every time: each replay here is followed by the program's own
eager work and a synchronisation, and the rounds fed to the replays differ."""
import numpy as np
import pytest

import kimad_synth as ks
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu

KW = dict(n_layer=2, vocab=4099)


def _outputs(plan, h):
    return [t.clone() for t in (plan.err_table, plan.j, plan.K, plan.offsets, plan.status, h)] + \
           [plan.idx[:int(plan.offsets[-1])].clone(), plan.val[:int(plan.offsets[-1])].clone()]


def _same(a, b):
    import torch
    return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a, b))


def test_step_on_a_stream_of_the_callers_equals_the_default_stream():
    import torch
    work = ks.make_workload("gpt2", **KW)
    g, h = gh.to_device(work)
    h0 = h.clone()
    plan = gh.make_plan(work, g, h)
    assert plan.step(work.budget_bytes).cpu().tolist() == [0, 0]
    torch.cuda.synchronize()
    ref = _outputs(plan, h)
    # against the oracle once, so that "equal" below means "right"
    E_gpu = plan.err_table.cpu().numpy().reshape(work.L, -1)
    st, j_ref, K_ref, off_ref = ko.allocate(E_gpu, plan.grid_sizes(), work.budget_bytes, 8, work.cost_units_D)
    assert st == ko.OK and np.array_equal(plan.K.cpu().numpy().astype(np.uint64), K_ref)
    gh.check_compress(work, plan, h, K_ref, off_ref, plan.idx, plan.val)

    s = torch.cuda.Stream()
    for _ in range(2):                       # the second one predicts from the first one's histogram
        h.copy_(h0)
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            plan.step(work.budget_bytes)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        assert _same(_outputs(plan, h), ref)


def test_step_recorded_into_a_graph_replays_like_eager_calls():
    import torch
    rounds = [ks.make_workload("gpt2", step=t, **KW) for t in range(3)]
    work = rounds[0]
    g, h = gh.to_device(work)
    plan = gh.make_plan(work, g, h)
    budgets = [work.budget_bytes, work.budget_bytes, work.budget_bytes]

    # eager reference: three rounds, the estimator carried over
    ref = []
    for t, w in enumerate(rounds):
        g.copy_(torch.from_numpy(w.g))
        assert plan.step(budgets[t]).cpu().tolist() == [0, 0]
        torch.cuda.synchronize()
        ref.append(_outputs(plan, h))

    # record one step (the plan has a histogram to predict from by now, as in a running job)
    h.copy_(torch.from_numpy(work.h))
    g.copy_(torch.from_numpy(rounds[0].g))
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        plan.step(budgets[0])
    torch.cuda.synchronize()

    # an unrelated plan doing eager work between the replays
    other_w = ks.make_workload("resnet18")
    og, oh = gh.to_device(other_w)
    other = gh.make_plan(other_w, og, oh)

    for rep in range(2):                     # the chain twice over: six replays
        h.copy_(torch.from_numpy(work.h))
        for t, w in enumerate(rounds):
            g.copy_(torch.from_numpy(w.g))
            graph.replay()
            torch.cuda.synchronize()
            assert _same(_outputs(plan, h), ref[t]), (rep, t)
            assert other.step(other_w.budget_bytes).cpu().tolist() == [0, 0]
            x = (og * 2.0).sum()
            torch.cuda.synchronize()
            assert bool(torch.isfinite(x))
