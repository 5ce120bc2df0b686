"""Whole rounds of Algorithm 1 on the GPU, both directions, against the oracle bit for bit: workers
compress u_m - u_hat_m under the up-link budget, the server decodes and steps the model, then
compresses x - x_hat under the down-link budget with the same library (Section 3.1: bidirectional
compression), and the workers decode that into their copy of the model estimator.  Budgets follow
Eq. budget on the sin^2 bandwidth pattern of Section 4.2."""
import numpy as np
import pytest

import kimad_synth as ks
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def test_three_rounds_two_workers_both_directions():
    import torch
    import paper_2312_08053_amd as kimad
    M, rounds, gamma, t_step, t_comp = 2, 3, 0.05, 0.02, 0.004
    base = ks.make_workload("mlp")
    sizes, ratios, d, L = base.sizes, base.ratios, base.d, base.L
    starts_np = np.asarray(base.starts, dtype=np.int64)
    starts = torch.from_numpy(starts_np).cuda()
    times = np.arange(rounds) * 20.0
    bw_up = [ks.sin2_bandwidth_trace(times, noise=0.1, seed=m) for m in range(M)]
    bw_down = ks.sin2_bandwidth_trace(times + 7.0)
    rng = np.random.default_rng(4)
    x_ref = rng.standard_normal(d).astype(np.float32) * np.float32(0.1)
    xhat_ref = np.zeros(d, np.float32)
    uhat_ref = [np.zeros(d, np.float32) for _ in range(M)]

    # device state: each worker's estimator (worker copy and server copy), the model, the model
    # estimator (server copy and one worker's copy)
    x = torch.from_numpy(x_ref.copy()).cuda()
    xhat_s = torch.zeros(d, dtype=torch.float32, device="cuda")
    xhat_w = torch.zeros(d, dtype=torch.float32, device="cuda")
    g = [torch.zeros(d, dtype=torch.float32, device="cuda") for _ in range(M)]
    uhat_w = [torch.zeros(d, dtype=torch.float32, device="cuda") for _ in range(M)]
    uhat_s = [torch.zeros(d, dtype=torch.float32, device="cuda") for _ in range(M)]
    cap = 4 * d
    plans = [kimad.Plan(g[m], uhat_w[m], sizes.tolist(), ratios.tolist(), max_budget_bytes=cap) for m in range(M)]
    down = kimad.Plan(x, xhat_s, sizes.tolist(), ratios.tolist(), max_budget_bytes=cap)

    def layers(a):
        return [a[starts_np[i]:starts_np[i + 1]] for i in range(L)]

    def oracle_step(plan, g_np, h_np, budget):
        """The oracle on the same inputs; the allocation on the library's own error table, which the
        oracle's table only matches to 1e-5 (a near-tie could otherwise pick another K)."""
        E_ref, Kt = ko.profile(layers(g_np), layers(h_np), ratios)
        E_gpu = plan.err_table.cpu().numpy().reshape(L, -1)
        gh.assert_table_close(E_gpu, E_ref, Kt, sizes)
        st, _, K, off = ko.allocate(E_gpu, Kt, budget, 8, 0)
        assert st == ko.OK
        off2, idx, val, h_new = ko.compress_ef(layers(g_np), layers(h_np), K)
        assert np.array_equal(off, off2) and 8 * int(off[-1]) <= budget
        n = int(off[-1])
        assert np.array_equal(plan.offsets.cpu().numpy().astype(np.uint64), off)
        assert np.array_equal(gh.u32(plan.idx)[:n], idx)
        assert np.array_equal(plan.val.cpu().numpy()[:n].view(np.uint32), val.view(np.uint32))
        return (off, idx, val), np.concatenate(h_new)

    for k in range(rounds):
        payloads_ref, payloads = [], []
        before = [a.copy() for a in uhat_ref]
        for m in range(M):
            u = ks.make_workload("mlp", seed=10 + m, step=k).g
            g[m].copy_(torch.from_numpy(u))
            budget = kimad.kimad_budget_bytes(bw_up[m][k], t_step, t_comp, 1.0, cap)
            assert budget == ko.budget_bytes(bw_up[m][k], t_step, t_comp, 1.0, cap) and budget >= 8 * L
            assert plans[m].step(budget).cpu().tolist() == [0, 0]
            pl, uhat_ref[m] = oracle_step(plans[m], u, before[m], budget)
            payloads_ref.append(pl)
            payloads.append((plans[m].idx, plans[m].val, plans[m].offsets))
        # server: decode every worker's payload into its copy of that worker's estimator, step the model
        kimad.kimad_server_apply(payloads, uhat_s, [1.0 / M] * M, starts, d, x, gamma)
        hats, x_ref = ko.server_apply(payloads_ref, before, [1.0 / M] * M, x_ref, gamma, starts_np)
        torch.cuda.synchronize()
        for m in range(M):
            assert np.array_equal(hats[m].view(np.uint32), uhat_ref[m].view(np.uint32))
            assert torch.equal(uhat_s[m], uhat_w[m]), "server and worker copies of an estimator stay equal"
            assert np.array_equal(uhat_s[m].cpu().numpy().view(np.uint32), uhat_ref[m].view(np.uint32))
        assert np.array_equal(x.cpu().numpy().view(np.uint32), x_ref.view(np.uint32))
        # down-link: the same library on x - x_hat, decoded by the worker with the server-side call
        budget = kimad.kimad_budget_bytes(bw_down[k], t_step, t_comp, 1.0, cap)
        assert down.step(budget).cpu().tolist() == [0, 0]
        _, xhat_ref = oracle_step(down, x_ref, xhat_ref, budget)
        kimad.kimad_server_apply([(down.idx, down.val, down.offsets)], [xhat_w], [1.0], starts, d)
        torch.cuda.synchronize()
        assert torch.equal(xhat_w, xhat_s), "worker and server copies of the model estimator stay equal"
        assert np.array_equal(xhat_s.cpu().numpy().view(np.uint32), xhat_ref.view(np.uint32))


def test_quadratic_single_worker_up_link_only_converges_like_the_oracle():
    """The setting of the synthetic experiments (Section 4.1): one worker, f(x) = 1/2 sum a_i x_i^2 with
    d = 30, the down-link free, the up-link budget following the sin^2 bandwidth pattern, layer-wise
    EF21 around the compressor.  Here the 30 coordinates are three layers of 10 so that the allocation
    has something to decide.  Every round's payload, estimator and model must equal the oracle's bit
    for bit, and the method must converge: f falls by more than six orders of magnitude."""
    import torch
    import paper_2312_08053_amd as kimad
    d, L, rounds, gamma = 30, 3, 400, np.float32(0.25)
    sizes = np.full(L, d // L, dtype=np.int64)
    starts_np = np.arange(L + 1, dtype=np.int64) * (d // L)
    starts = torch.from_numpy(starts_np).cuda()
    ratios = np.arange(1, 11) / 10.0
    a = np.linspace(0.2, 1.0, d).astype(np.float32)
    x_ref = np.ones(d, np.float32)
    uhat_ref = np.zeros(d, np.float32)
    # up to 12 pairs a round at the crest of the pattern, 3 (one per layer) in the trough
    bw = ks.sin2_bandwidth_trace(np.arange(rounds) * 3.0, eta=72.0 * 8, theta=0.05, delta=24.0 * 8)
    x = torch.from_numpy(x_ref.copy()).cuda()
    g = torch.zeros(d, dtype=torch.float32, device="cuda")
    uhat_w = torch.zeros(d, dtype=torch.float32, device="cuda")
    uhat_s = torch.zeros(d, dtype=torch.float32, device="cuda")
    plan = kimad.Plan(g, uhat_w, sizes.tolist(), ratios.tolist(), max_budget_bytes=8 * d)

    def layers(v):
        return [v[starts_np[i]:starts_np[i + 1]] for i in range(L)]

    f0 = 0.5 * float(np.sum(a.astype(np.float64) * x_ref.astype(np.float64) ** 2))
    seen = set()
    for k in range(rounds):
        u = a * x_ref                                           # the worker's gradient at the model it holds
        g.copy_(torch.from_numpy(u))
        budget = kimad.kimad_budget_bytes(float(bw[k]), 1.0, 0.0, 0.0, 8 * d)
        assert budget == ko.budget_bytes(float(bw[k]), 1.0, 0.0, 0.0, 8 * d) and budget >= 8 * L
        seen.add(budget // 8)
        assert plan.step(budget).cpu().tolist() == [0, 0], k
        E_ref, Kt = ko.profile(layers(u), layers(uhat_ref), ratios)
        gh.assert_table_close(plan.err_table.cpu().numpy().reshape(L, -1), E_ref, Kt, sizes)
        st, _, K, off = ko.allocate(plan.err_table.cpu().numpy().reshape(L, -1), Kt, budget, 8, 0)
        assert st == ko.OK and np.array_equal(plan.K.cpu().numpy().astype(np.uint64), K)
        off2, idx, val, h_new = ko.compress_ef(layers(u), layers(uhat_ref), K)
        n = int(off[-1])
        assert np.array_equal(gh.u32(plan.idx)[:n], idx), k
        assert np.array_equal(plan.val.cpu().numpy()[:n].view(np.uint32), val.view(np.uint32)), k
        kimad.kimad_server_apply([(plan.idx, plan.val, plan.offsets)], [uhat_s], [1.0], starts, d, x, float(gamma))
        hats, x_ref = ko.server_apply([(off, idx, val)], [uhat_ref], [1.0], x_ref, float(gamma), starts_np)
        uhat_ref = np.concatenate(h_new)
        torch.cuda.synchronize()
        assert np.array_equal(hats[0].view(np.uint32), uhat_ref.view(np.uint32))
        assert torch.equal(uhat_s, uhat_w)
        assert np.array_equal(uhat_s.cpu().numpy().view(np.uint32), uhat_ref.view(np.uint32)), k
        assert np.array_equal(x.cpu().numpy().view(np.uint32), x_ref.view(np.uint32)), k
    assert len(seen) >= 6, "the budget must really vary over the rounds"
    f_end = 0.5 * float(np.sum(a.astype(np.float64) * x_ref.astype(np.float64) ** 2))
    assert f_end < 1e-6 * f0, (f0, f_end)


def test_allocation_from_the_previous_rounds_profile():
    """Profile and allocation may run while the previous round is still on the wire, one round late
    (the overlap Section 5 points at): round k is then compressed with the K chosen from round k-1's
    error table.  The compression must not look at anything the stale profile left behind: payload
    and estimator equal the oracle's for the same K, and the payload still fits the budget."""
    import torch
    w0 = ks.make_workload("llama", n_layer=1, hidden=512, ffn=1408, vocab=3001, step=0)
    g = torch.from_numpy(w0.g).cuda()
    h = torch.from_numpy(w0.h).cuda()
    plan = gh.make_plan(w0, g, h)
    h_ref = [v.copy() for v in w0.layer_views(w0.h)]
    K_ref = None
    for k in range(4):
        wk = ks.make_workload("llama", n_layer=1, hidden=512, ffn=1408, vocab=3001, step=k)
        g.copy_(torch.from_numpy(wk.g))
        gL = wk.layer_views(wk.g)
        if K_ref is not None:
            # K and offsets of the previous round's allocation are still in plan.K / plan.offsets
            plan.compress_ef(reuse_profile=False)
            torch.cuda.synchronize()
            assert plan.status.cpu().tolist()[1] == 0
            off, idx, val, h_new = ko.compress_ef(gL, h_ref, K_ref)
            n = int(off[-1])
            assert w0.pair_bytes * n <= w0.budget_bytes
            assert np.array_equal(plan.offsets.cpu().numpy().astype(np.uint64), off)
            assert np.array_equal(gh.u32(plan.idx)[:n], idx), k
            assert np.array_equal(plan.val.cpu().numpy()[:n].view(np.uint32), val.view(np.uint32)), k
            assert np.array_equal(h.cpu().numpy().view(np.uint32), np.concatenate(h_new).view(np.uint32)), k
            h_ref = h_new
        # this round's profile (of g_k - h after the update) decides the next round's K
        plan.profile(budget_hint_bytes=w0.budget_bytes)
        plan.allocate(w0.budget_bytes)
        torch.cuda.synchronize()
        assert plan.status.cpu().tolist()[0] == 0
        E_ref, Kt = ko.profile(gL, h_ref, w0.ratios)
        E_gpu = plan.err_table.cpu().numpy().reshape(w0.L, -1)
        gh.assert_table_close(E_gpu, E_ref, Kt, w0.sizes)
        st, _, K_ref, _ = ko.allocate(E_gpu, Kt, w0.budget_bytes, w0.pair_bytes, w0.cost_units_D)
        assert st == ko.OK and np.array_equal(plan.K.cpu().numpy().astype(np.uint64), K_ref)
