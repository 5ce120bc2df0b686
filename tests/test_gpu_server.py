"""GPU parity of the server step (Algorithm 1: aggregate the estimators, update the model): bit for bit."""
import numpy as np
import pytest

import kimad_synth as ks
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _dev_payload(offsets, idx, val):
    import torch
    return (torch.from_numpy(idx.astype(np.uint32).view(np.int32)).cuda(),
            torch.from_numpy(val.astype(np.float32)).cuda(),
            torch.from_numpy(offsets.astype(np.int64)).cuda())


def test_round_trip_worker_on_gpu_then_server_on_gpu():
    # the worker compresses on the GPU; the server decodes that payload on the GPU into its own copy
    # of the estimator, which must then equal the worker's, and steps the model
    import torch
    import paper_2312_08053_amd as kimad
    work = ks.make_workload("resnet18")
    g, h = gh.to_device(work)
    server_hat = h.clone()
    plan = gh.make_plan(work, g, h)
    assert plan.step(work.budget_bytes).cpu().tolist() == [0, 0]
    starts = torch.from_numpy(np.asarray(work.starts, dtype=np.int64)).cuda()
    rng = np.random.default_rng(11)
    x0 = rng.standard_normal(work.d).astype(np.float32)
    x = torch.from_numpy(x0).cuda()
    kimad.kimad_server_apply([(plan.idx, plan.val, plan.offsets)], [server_hat], [1.0], starts, work.d, x, 0.05)
    torch.cuda.synchronize()
    assert torch.equal(server_hat, h), "server and worker estimators must stay equal bit for bit"
    off = plan.offsets.cpu().numpy().astype(np.uint64)
    hats, x1 = ko.server_apply([(off, gh.u32(plan.idx), plan.val.cpu().numpy())], [work.h], [1.0], x0, 0.05, work.starts)
    assert np.array_equal(server_hat.cpu().numpy().view(np.uint32), hats[0].view(np.uint32))
    assert np.array_equal(x.cpu().numpy().view(np.uint32), x1.view(np.uint32))


@pytest.mark.parametrize("M", [1, 3, 16])
def test_several_workers_against_the_oracle(M):
    import torch
    import paper_2312_08053_amd as kimad
    sizes = [40001, 7, 8192, 1023, 16385]
    starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    d = int(starts[-1])
    rng = np.random.default_rng(100 + M)
    pls, hats, w = [], [], []
    for m in range(M):
        g = [rng.standard_normal(n).astype(np.float32) * np.float32(10.0 ** rng.uniform(-3, 2)) for n in sizes]
        h = [(0.5 * rng.standard_normal(n)).astype(np.float32) for n in sizes]
        K = np.array([rng.integers(0, n + 1) for n in sizes], dtype=np.uint64)     # 0 and n included now and then
        if m == 0:
            K[1] = 0
            K[3] = sizes[3]
        offsets, idx, val, _ = ko.compress_ef(g, h, K)
        pls.append((offsets, idx, val))
        hats.append(np.concatenate(h))
        w.append(float(rng.uniform(0.0, 1.0)))
    x0 = rng.standard_normal(d).astype(np.float32)
    gamma = 0.37
    ref_hats, ref_x = ko.server_apply(pls, hats, w, x0, gamma, starts)
    dev_hats = [torch.from_numpy(u.copy()).cuda() for u in hats]
    x = torch.from_numpy(x0.copy()).cuda()
    kimad.kimad_server_apply([_dev_payload(*p) for p in pls], dev_hats, w, torch.from_numpy(starts).cuda(), d, x, gamma)
    torch.cuda.synchronize()
    for m in range(M):
        assert np.array_equal(dev_hats[m].cpu().numpy().view(np.uint32), ref_hats[m].view(np.uint32)), m
    assert np.array_equal(x.cpu().numpy().view(np.uint32), ref_x.view(np.uint32))


def test_aggregate_only_and_unaligned_buffers():
    # x = NULL leaves the model alone; buffers that start off a 16-byte boundary take the scalar path
    import torch
    import paper_2312_08053_amd as kimad
    sizes = [1001, 64]
    starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    d = int(starts[-1])
    rng = np.random.default_rng(5)
    g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    h = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    offsets, idx, val, h_new = ko.compress_ef(g, h, np.array([100, 64], dtype=np.uint64))
    big = torch.zeros(d + 8, dtype=torch.float32, device="cuda")
    u = big[1:1 + d]                                    # 4 bytes past a 16-byte boundary
    u.copy_(torch.from_numpy(np.concatenate(h)))
    st = torch.from_numpy(starts).cuda()
    kimad.kimad_server_apply([_dev_payload(offsets, idx, val)], [u], [1.0], st, d, None, 0.0)
    torch.cuda.synchronize()
    assert np.array_equal(u.cpu().numpy().view(np.uint32), np.concatenate(h_new).view(np.uint32))
    xb = torch.zeros(d + 8, dtype=torch.float32, device="cuda")
    x = xb[3:3 + d]
    x0 = rng.standard_normal(d).astype(np.float32)
    x.copy_(torch.from_numpy(x0))
    empty = (np.zeros(len(sizes) + 1, np.uint64), np.zeros(1, np.uint32), np.zeros(1, np.float32))
    kimad.kimad_server_apply([_dev_payload(*empty)], [u], [0.25], st, d, x, 2.0)
    torch.cuda.synchronize()
    _, want = ko.server_apply([(empty[0], empty[1][:0], empty[2][:0])], [np.concatenate(h_new)], [0.25], x0, 2.0, starts)
    assert np.array_equal(x.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_server_apply_refuses_bad_arguments():
    import torch
    import paper_2312_08053_amd as kimad
    u = torch.zeros(8, device="cuda")
    st = torch.tensor([0, 8], dtype=torch.int64, device="cuda")
    pl = (torch.zeros(1, dtype=torch.int32, device="cuda"), torch.zeros(1, device="cuda"),
          torch.zeros(2, dtype=torch.int64, device="cuda"))
    with pytest.raises(kimad.KimadError):
        kimad.kimad_server_apply([pl] * 17, [u] * 17, [1.0] * 17, st, 8, None, 0.0)     # too many workers
    with pytest.raises(kimad.KimadError):
        kimad.kimad_server_apply([(None, pl[1], pl[2])], [u], [1.0], st, 8, None, 0.0)  # null pointer


def test_payloads_that_do_not_fit_the_layers_are_flagged_and_write_nothing_out_of_bounds():
    """The server's input comes from workers, not from this library: corrupted offsets or indices must end in a
    status, never in a write outside the estimator (guard words on both sides stay as they were)."""
    import torch
    import paper_2312_08053_amd as kimad
    sizes = np.array([10, 3, 50], dtype=np.int64)
    starts = np.concatenate([[0], np.cumsum(sizes)])
    d = int(starts[-1])
    st = torch.from_numpy(starts).cuda()
    guard = 16
    offsets = np.array([0, 2, 3, 6], dtype=np.int64)
    idx = np.array([1, 9, 2, 0, 7, 49], dtype=np.uint32)
    val = np.arange(1, 7, dtype=np.float32)

    def run(off_, idx_, cap_extra=0):
        buf = torch.full((d + 2 * guard,), 7.0, device="cuda")
        u = buf[guard:guard + d]
        u.zero_()
        i_t = torch.from_numpy(np.concatenate([idx_, np.zeros(cap_extra, np.uint32)]).view(np.int32)).cuda()
        v_t = torch.from_numpy(np.concatenate([val[:len(idx_)], np.zeros(cap_extra, np.float32)])).cuda()
        o_t = torch.from_numpy(off_).cuda()
        status = kimad.kimad_server_apply([(i_t, v_t, o_t)], [u], [1.0], st, d, None, 0.0)
        torch.cuda.synchronize()
        b = buf.cpu().numpy()
        assert np.all(b[:guard] == 7.0) and np.all(b[guard + d:] == 7.0)
        return int(status.item()), b[guard:guard + d]

    code, u = run(offsets, idx)
    want = np.zeros(d, np.float32)
    for i in range(3):
        for p in range(offsets[i], offsets[i + 1]):
            want[starts[i] + idx[p]] += val[p]
    assert code == 0 and np.array_equal(u, want)
    bad_idx = idx.copy()
    bad_idx[2] = 3                                        # layer 1 has 3 entries: index 3 is outside it
    code, u = run(offsets, bad_idx)
    want2 = want.copy()
    want2[starts[1] + 2] = 0.0
    assert code == -13 and np.array_equal(u, want2)       # that pair skipped, the others applied
    bad_idx[5] = 0xFFFFFFF0
    code, u = run(offsets, bad_idx)
    assert code == -13
    for bad_off in (np.array([0, 4, 3, 6]), np.array([1, 2, 3, 6]), np.array([0, 2, 3, 1 << 40]), np.array([0, 2, 3, 7])):
        code, u = run(bad_off.astype(np.int64), idx)
        assert code == -13 and not u.any(), bad_off       # nothing of such a payload is applied
    # layer starts that do not end at d
    st_bad = torch.from_numpy(np.array([0, 10, 13, 64], dtype=np.int64)).cuda()
    u = torch.zeros(d, device="cuda")
    status = kimad.kimad_server_apply([_dev_payload(offsets, idx, val)], [u], [1.0], st_bad, d, None, 0.0)
    assert int(status.item()) == -13 and not u.cpu().numpy().any()
