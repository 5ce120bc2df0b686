"""Pins of the oracle's server step (Algorithm 1: aggregate the estimators, update the model)."""
from fractions import Fraction

import numpy as np

from oracle import kimad_oracle as ko


def _worker(seed, sizes, ratio=0.25):
    rng = np.random.default_rng(seed)
    g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    h = [(0.3 * rng.standard_normal(n)).astype(np.float32) for n in sizes]
    K = np.array([max(1, int(np.ceil(ratio * n))) for n in sizes], dtype=np.uint64)
    return g, h, K


def _starts(sizes):
    return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)


def test_server_estimator_equals_the_workers_after_decoding():
    # the server's copy of u_hat_m must track the worker's bit for bit (Algorithm 1 keeps both)
    sizes = [37, 1, 300, 64]
    g, h, K = _worker(1, sizes)
    offsets, idx, val, h_new = ko.compress_ef(g, h, K)
    hats, x = ko.server_apply([(offsets, idx, val)], [np.concatenate(h)], [1.0], None, 0.0, _starts(sizes))
    assert x is None
    assert np.array_equal(hats[0].view(np.uint32), np.concatenate(h_new).view(np.uint32))


def test_full_payload_from_zero_estimator_gives_plain_sgd_step():
    # K = n and u_hat = 0: the estimator becomes the update itself and x_new = fl32(x - gamma * g)
    sizes = [5, 12]
    rng = np.random.default_rng(2)
    g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    h = [np.zeros(n, np.float32) for n in sizes]
    offsets, idx, val, _ = ko.compress_ef(g, h, np.array(sizes, dtype=np.uint64))
    x0 = rng.standard_normal(sum(sizes)).astype(np.float32)
    gamma = 0.125
    hats, x1 = ko.server_apply([(offsets, idx, val)], [np.concatenate(h)], [1.0], x0, gamma, _starts(sizes))
    gflat = np.concatenate(g)
    assert np.array_equal(hats[0], gflat)
    want = np.array([np.float32(float(a) - gamma * float(b)) for a, b in zip(x0, gflat)], dtype=np.float32)
    assert np.array_equal(x1.view(np.uint32), want.view(np.uint32))


def test_model_step_against_exact_rationals():
    # small dyadic values: every product and sum below is exact in fp64, so the result must equal
    # the correctly rounded exact value
    sizes = [6, 3]
    M = 3
    rng = np.random.default_rng(3)
    hats = [(rng.integers(-64, 64, size=sum(sizes)) / 16.0).astype(np.float32) for _ in range(M)]
    empty = (np.zeros(len(sizes) + 1, np.uint64), np.zeros(0, np.uint32), np.zeros(0, np.float32))
    w = [0.5, 0.25, 0.25]
    gamma = 0.375
    x0 = (rng.integers(-1024, 1024, size=sum(sizes)) / 64.0).astype(np.float32)
    new_hats, x1 = ko.server_apply([empty] * M, hats, w, x0, gamma, _starts(sizes))
    for m in range(M):
        assert np.array_equal(new_hats[m], hats[m])          # empty payloads change nothing
    for t in range(sum(sizes)):
        exact = Fraction(float(x0[t])) - Fraction(gamma) * sum(Fraction(w[m]) * Fraction(float(hats[m][t])) for m in range(M))
        assert Fraction(float(x1[t])) == exact               # representable: no rounding at all here


def test_zero_step_size_and_zero_weights_leave_the_model():
    sizes = [9]
    g, h, K = _worker(4, sizes)
    pl = ko.compress_ef(g, h, K)[:3]
    x0 = np.arange(9, dtype=np.float32)
    _, xa = ko.server_apply([pl], [np.concatenate(h)], [1.0], x0, 0.0, _starts(sizes))
    _, xb = ko.server_apply([pl], [np.concatenate(h)], [0.0], x0, 0.7, _starts(sizes))
    assert np.array_equal(xa, x0) and np.array_equal(xb, x0)


def test_decoding_touches_only_the_support_and_the_right_layer():
    sizes = [4, 4]
    h = [np.zeros(4, np.float32), np.zeros(4, np.float32)]
    offsets = np.array([0, 1, 3], dtype=np.uint64)
    idx = np.array([2, 0, 3], dtype=np.uint32)               # layer 0: {2}; layer 1: {0, 3}
    val = np.array([1.5, -2.0, 4.0], dtype=np.float32)
    hats, _ = ko.server_apply([(offsets, idx, val)], [np.concatenate(h)], [1.0], None, 0.0, _starts(sizes))
    assert hats[0].tolist() == [0, 0, 1.5, 0, -2.0, 0, 0, 4.0]


def test_two_workers_with_different_supports_average():
    sizes = [8]
    starts = _starts(sizes)
    pls, hs = [], []
    for seed in (5, 6):
        g, h, K = _worker(seed, sizes, ratio=0.5)
        pls.append(ko.compress_ef(g, h, K)[:3])
        hs.append(np.concatenate(h))
    x0 = np.zeros(8, np.float32)
    hats, x1 = ko.server_apply(pls, hs, [0.5, 0.5], x0, 1.0, starts)
    want = -(0.5 * hats[0].astype(np.float64) + 0.5 * hats[1].astype(np.float64))
    assert np.allclose(x1, want, rtol=0, atol=1e-7)


def test_model_step_precision_and_order_of_the_weighted_sum():
    # reading R13 evaluated with Python's own double arithmetic, term by term in worker order:
    # an fp32 accumulation or another summation order differs on these values
    M, n = 5, 200
    rng = np.random.default_rng(7)
    hats = [(rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32) for _ in range(M)]
    w = [1.0 / 3.0, 0.1, 0.2, 1.0 / 7.0, 0.05]
    gamma = 0.01
    x0 = rng.standard_normal(n).astype(np.float32)
    empty = (np.zeros(2, np.uint64), np.zeros(0, np.uint32), np.zeros(0, np.float32))
    _, x1 = ko.server_apply([empty] * M, hats, w, x0, gamma, [0, n])
    differs32 = 0
    for t in range(n):
        acc = 0.0
        acc32 = np.float32(0.0)
        for m in range(M):
            acc = acc + w[m] * float(hats[m][t])
            acc32 = np.float32(acc32 + np.float32(w[m]) * hats[m][t])
        want = np.float32(float(x0[t]) - gamma * acc)
        assert x1[t] == want
        differs32 += int(np.float32(x0[t] - np.float32(gamma) * acc32) != want)
    assert differs32 > 0          # the check can tell the two precisions apart
