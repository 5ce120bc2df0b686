"""Pins for the oracle's payload and estimator update (paper Section 3.3, Eq. EF21-2; Algorithm 1)."""
import numpy as np
import pytest

from oracle import kimad_oracle as ko


def test_by_hand_small_case():
    g = np.array([3.0, 1.0, 0.5, -2.0], dtype=np.float32)
    h = np.array([1.0, 4.0, 0.5, 0.0], dtype=np.float32)
    # x = [2, -3, 0, -2]; top-2 by magnitude: index 1 (3), then index 0 (|2| ties with index 3, lower wins)
    idx, val, hn = ko.compress_ef_layer(g, h, 2)
    assert idx.tolist() == [0, 1] and val.tolist() == [2.0, -3.0]
    assert hn.tolist() == [3.0, 1.0, 0.5, 0.0]
    idx, val, hn = ko.compress_ef_layer(g, h, 3)
    assert idx.tolist() == [0, 1, 3] and val.tolist() == [2.0, -3.0, -2.0]
    assert hn.tolist() == [3.0, 1.0, 0.5, -2.0]
    idx, val, hn = ko.compress_ef_layer(g, h, 0)
    assert idx.size == 0 and np.array_equal(hn, h)


@pytest.mark.parametrize("seed", range(5))
def test_server_and_worker_estimators_agree(seed):
    # Algorithm 1: the server adds the received compressed vector to its own copy of the
    # estimator; both copies must stay identical, bit for bit.
    rng = np.random.default_rng(seed)
    n = 3000 + seed
    g = (rng.standard_t(3, n) * 1e-2).astype(np.float32)
    h = (rng.standard_t(3, n) * 5e-3).astype(np.float32)
    for K in (1, 17, n // 3, n):
        idx, val, hn = ko.compress_ef_layer(g, h, K)
        assert idx.dtype == np.uint32 and val.dtype == np.float32 and hn.dtype == np.float32
        assert len(idx) == K and np.all(np.diff(idx.astype(np.int64)) > 0)
        server = h.copy()
        for t, v in zip(idx.tolist(), val.tolist()):              # scalar scatter-add, fp32
            server[t] = np.float32(server[t]) + np.float32(v)
        assert np.array_equal(server.view(np.uint32), hn.view(np.uint32))
        off = np.ones(n, bool)
        off[idx] = False
        assert np.array_equal(hn[off].view(np.uint32), h[off].view(np.uint32))
        assert np.array_equal(val.view(np.uint32), (g - h)[idx].view(np.uint32))


def test_zero_estimator_full_k_reproduces_g():
    rng = np.random.default_rng(3)
    g = rng.standard_normal(500).astype(np.float32)
    idx, val, hn = ko.compress_ef_layer(g, np.zeros_like(g), 500)
    assert idx.tolist() == list(range(500))
    assert np.array_equal(hn.view(np.uint32), g.view(np.uint32))


def test_update_is_h_plus_x_not_a_copy_of_g():
    # fl(h + fl(g - h)) need not equal g: the estimator follows Eq. EF21-2 literally.
    g = np.array([1.0], dtype=np.float32)
    h = np.array([1e-8], dtype=np.float32)
    # g - h rounds to 1 - 2^-24... check against arithmetic done on numpy scalars
    x = np.float32(g[0]) - np.float32(h[0])
    expect = np.float32(h[0]) + x
    idx, val, hn = ko.compress_ef_layer(g, h, 1)
    assert hn[0] == expect and val[0] == x
    rng = np.random.default_rng(5)
    g = rng.standard_normal(20000).astype(np.float32)
    h = (rng.standard_normal(20000) * 3).astype(np.float32)
    idx, val, hn = ko.compress_ef_layer(g, h, 20000)
    assert np.any(hn != g)                                       # the distinction is observable
    assert np.array_equal(hn, h + (g - h))


def test_multi_layer_payload_layout_and_step_budget():
    rng = np.random.default_rng(8)
    sizes = [10, 257, 1, 64]
    g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    h = [rng.standard_normal(n).astype(np.float32) * 0.3 for n in sizes]
    K = [3, 100, 1, 0]
    off, idx, val, hn = ko.compress_ef(g, h, K)
    assert off.tolist() == [0, 3, 103, 104, 104]
    for i in range(4):
        a, b = int(off[i]), int(off[i + 1])
        li, lv, lh = ko.compress_ef_layer(g[i], h[i], K[i])
        assert np.array_equal(idx[a:b], li) and np.array_equal(val[a:b], lv) and np.array_equal(hn[i], lh)
        assert np.all(idx[a:b] < sizes[i])
    ratios = [0.05, 0.2, 0.5, 1.0]
    for budget in (8 * 20, 8 * 100, 8 * 400):
        out = ko.step(g, h, ratios, budget, 8, 0)
        assert out["status"] == ko.OK
        assert 8 * len(out["idx"]) <= budget                     # Eq. optimisation, the constraint
        # the step's error equals the profile's prediction for the chosen sizes
        for i in range(4):
            x = g[i] - h[i]
            resid = x.astype(np.float64).copy()
            a, b = int(out["offsets"][i]), int(out["offsets"][i + 1])
            resid[out["idx"][a:b]] = 0.0
            assert float((resid ** 2).sum()) == pytest.approx(out["E"][i, out["j"][i]], rel=1e-12, abs=1e-300)
