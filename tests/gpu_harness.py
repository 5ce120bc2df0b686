"""Helpers shared by the GPU parity tests: run the library on a workload, run the oracle, compare."""
from __future__ import annotations

import numpy as np

from oracle import kimad_oracle as ko


def to_device(work):
    import torch
    g = torch.from_numpy(work.g).cuda()
    h = torch.from_numpy(work.h).cuda()
    return g, h


def make_plan(work, g, h, **kw):
    import paper_2312_08053_amd as kimad
    args = dict(pair_bytes=work.pair_bytes, D=work.cost_units_D, max_budget_bytes=max(work.budget_bytes, 8))
    args.update(kw)
    return kimad.Plan(g, h, work.sizes.tolist(), work.ratios.tolist(), **args)


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def assert_table_close(E_gpu: np.ndarray, E_ref: np.ndarray, Kt: np.ndarray, sizes, rel=1e-5):
    """Error-table parity: exactly 0 where K = n, otherwise within `rel` relative (fp32-grade bar)."""
    E_gpu = E_gpu.reshape(E_ref.shape)
    full = Kt == np.asarray(sizes, dtype=np.int64)[:, None]
    assert np.all(E_gpu[full] == 0.0), "entries with K = n must be exactly zero"
    assert np.all(E_ref[full] == 0.0)
    fin = np.isfinite(E_ref)
    assert np.array_equal(np.isnan(E_gpu), np.isnan(E_ref))
    assert np.array_equal(np.isinf(E_gpu), np.isinf(E_ref))
    a, b = E_gpu[fin], E_ref[fin]
    bad = np.abs(a - b) > rel * np.abs(b)
    if bad.any():
        w = np.argwhere((np.abs(E_gpu - E_ref) > rel * np.abs(E_ref)) & fin)
        i, j = w[0]
        raise AssertionError(f"{bad.sum()} table entries off; first at layer {i} j {j}: "
                             f"gpu {E_gpu[i, j]!r} ref {E_ref[i, j]!r} K {Kt[i, j]} n {sizes[i]}")


def oracle_layers(work):
    return work.layer_views(work.g), work.layer_views(work.h)


def check_compress(work, plan, h_dev, K, offsets, idx_t, val_t, layers=None):
    """Payload and estimator against the oracle, bit for bit, for the given layers (default all)."""
    gL, hL = oracle_layers(work)
    idx = u32(idx_t)
    val = val_t.cpu().numpy().view(np.uint32)
    h_new = h_dev.cpu().numpy()
    starts = work.starts
    which = range(work.L) if layers is None else layers
    for i in which:
        li, lv, lh = ko.compress_ef_layer(gL[i], hL[i], int(K[i]))
        a, b = int(offsets[i]), int(offsets[i + 1])
        assert b - a == int(K[i])
        assert np.array_equal(idx[a:b], li), f"layer {i}: indices differ (n={work.sizes[i]}, K={K[i]})"
        assert np.array_equal(val[a:b], lv.view(np.uint32)), f"layer {i}: values differ"
        got = h_new[starts[i]:starts[i + 1]]
        assert np.array_equal(got.view(np.uint32), lh.view(np.uint32)), f"layer {i}: estimator differs"
