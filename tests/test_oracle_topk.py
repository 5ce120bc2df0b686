"""Pins for the oracle's TopK support and error profile.

Everything here is checked against something other than the oracle's own
formula: exhaustive search over subsets with exact rational arithmetic, closed
forms, numpy's partition, and the inequalities the paper's compressor class obeys.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import kimad_oracle as ko


def exact_drop_error(x, keep):
    """||x - x restricted to keep||^2 as an exact rational."""
    keep = set(keep)
    return sum((Fraction(float(v)) ** 2 for t, v in enumerate(x) if t not in keep), Fraction(0))


@pytest.mark.parametrize("seed", range(6))
def test_support_is_the_unique_minimiser_when_magnitudes_differ(seed):
    # Section 2.2: TopK keeps the K entries of largest absolute value, which is the
    # size-K support of least squared error.  Search every subset.
    rng = np.random.default_rng(seed)
    d = int(rng.integers(1, 9))
    x = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32)
    assert len(set(np.abs(x).tolist())) == d
    for K in range(1, d + 1):
        errs = {S: exact_drop_error(x, S) for S in itertools.combinations(range(d), K)}
        best = min(errs.values())
        winners = [S for S, e in errs.items() if e == best]
        assert len(winners) == 1
        got = tuple(sorted(ko.topk_support(x, K).tolist()))
        assert got == winners[0]
        E = ko.topk_error_profile(x, [K])[0]
        assert E == pytest.approx(float(best), rel=1e-14, abs=0.0)


@pytest.mark.parametrize("seed", range(6))
def test_support_is_a_minimiser_and_lowest_index_under_ties(seed):
    rng = np.random.default_rng(100 + seed)
    d = int(rng.integers(2, 9))
    x = rng.integers(-2, 3, size=d).astype(np.float32)          # many equal magnitudes
    for K in range(1, d + 1):
        errs = {S: exact_drop_error(x, S) for S in itertools.combinations(range(d), K)}
        best = min(errs.values())
        winners = [S for S, e in errs.items() if e == best]
        got = tuple(sorted(ko.topk_support(x, K).tolist()))
        assert got in winners
        # Among all minimisers the oracle's is the one that, magnitude class by magnitude
        # class, takes the lowest indices: i.e. the lexicographically smallest after
        # sorting candidates by (magnitude descending, index ascending).
        def rank_key(S):
            return sorted((-abs(float(x[t])), t) for t in S)
        assert rank_key(got) == min(rank_key(S) for S in winners)


def test_tie_rule_by_hand():
    x = np.array([1.0, -1.0, 1.0, 2.0, -1.0], dtype=np.float32)
    assert ko.topk_support(x, 1).tolist() == [3]
    assert ko.topk_support(x, 2).tolist() == [3, 0]
    assert ko.topk_support(x, 3).tolist() == [3, 0, 1]
    assert ko.topk_support(x, 4).tolist() == [3, 0, 1, 2]
    # errors: dropping three / two / one / no entries of magnitude 1 ...
    assert ko.topk_error_profile(x, [1, 2, 3, 4, 5]).tolist() == [4.0, 3.0, 2.0, 1.0, 0.0]


def test_signed_zero_denormal_inf_nan_order():
    den = np.float32(1e-45)                       # smallest denormal
    x = np.array([0.0, -0.0, den, -den, np.inf, -np.inf, np.nan, 1.0], dtype=np.float32)
    order = ko.magnitude_order(x).tolist()
    # NaN patterns rank above Inf, both infinities tie (index order), then 1, the
    # denormals tie, the two zeros tie.
    assert order == [6, 4, 5, 7, 2, 3, 0, 1]
    key = ko.magnitude_key(x)
    assert key[0] == key[1] == 0 and key[2] == key[3] == 1


@pytest.mark.parametrize("seed", range(4))
def test_matches_numpy_partition_as_a_set(seed):
    rng = np.random.default_rng(200 + seed)
    n = 1000 + 37 * seed
    x = rng.standard_t(3, n).astype(np.float32)
    assert len(np.unique(np.abs(x))) == n
    for K in (1, 2, n // 7, n // 2, n - 1, n):
        ref = set(np.argpartition(-np.abs(x), K - 1)[:K].tolist())
        assert set(ko.topk_support(x, K).tolist()) == ref


@pytest.mark.parametrize("seed", range(4))
def test_error_equals_sum_of_dropped_squares(seed):
    # Section 3.2, Eq. norm decomposition, recomputed without the oracle's ordering:
    # sort the squares, add the n-K smallest with exact summation.
    rng = np.random.default_rng(300 + seed)
    n = 4097 + seed
    x = (rng.laplace(0, 1, n) * 1e-3).astype(np.float32)
    Ks = [1, 5, n // 10, n // 2, n - 2, n - 1, n]
    E = ko.topk_error_profile(x, Ks)
    sq = np.sort(x.astype(np.float64) ** 2)
    for K, e in zip(Ks, E):
        ref = math.fsum(sq[: n - K].tolist())
        assert e == pytest.approx(ref, rel=1e-13, abs=0.0)
    assert E[-1] == 0.0


def test_constant_vector_closed_form():
    v = np.float32(0.375)
    d = 50
    x = np.full(d, v, dtype=np.float32)
    x[::2] *= -1
    Ks = list(range(1, d + 1))
    E = ko.topk_error_profile(x, Ks)
    assert E.tolist() == [(d - K) * float(v) ** 2 for K in Ks]
    for K in Ks:
        assert sorted(ko.topk_support(x, K).tolist()) == list(range(K))


@pytest.mark.parametrize("seed", range(4))
def test_monotone_zero_at_full_and_contraction_bound(seed):
    # Compressor class C(alpha) of the paper's appendix (definition of the contractive
    # class): ||C(x) - x||^2 <= (1 - alpha) ||x||^2, and TopK has alpha = K/d.
    rng = np.random.default_rng(400 + seed)
    n = 777
    x = (rng.standard_t(2.5, n) * 10.0 ** rng.uniform(-5, -1)).astype(np.float32)
    Ks = list(range(1, n + 1))
    E = ko.topk_error_profile(x, Ks)
    assert np.all(np.diff(E) <= 0.0)
    assert E[-1] == 0.0
    nrm = math.fsum((x.astype(np.float64) ** 2).tolist())
    for K, e in zip(Ks, E):
        assert e <= (1.0 - K / n) * nrm * (1 + 1e-12)


def test_single_element_layer():
    x = np.array([-3.5], dtype=np.float32)
    assert ko.topk_support(x, 1).tolist() == [0]
    assert ko.topk_error_profile(x, [1]).tolist() == [0.0]


def test_operand_is_g_minus_h_in_fp32():
    g = np.array([3.0, 1.0, 1e8], dtype=np.float32)
    h = np.array([1.0, 4.0, 1.0], dtype=np.float32)
    x = ko.operand(g, h)
    assert x.dtype == np.float32
    assert x.tolist() == [2.0, -3.0, 1e8]           # 1e8 - 1 rounds back to 1e8 in binary32


def test_grid_sizes_by_hand():
    r = [0.001, 0.05, 0.1, 0.11, 0.5, 0.99, 1.0]
    assert ko.grid_sizes(r, 10).tolist() == [1, 1, 1, 2, 5, 10, 10]
    assert ko.grid_sizes(r, 1).tolist() == [1] * 7
    assert ko.grid_sizes(r, 1000).tolist() == [1, 50, 100, 110, 500, 990, 1000]
    assert ko.grid_sizes([0.3], 7).tolist() == [3]   # ceil(2.1)


def test_profile_table_rows_are_independent_layers():
    rng = np.random.default_rng(9)
    g = [rng.standard_normal(n).astype(np.float32) for n in (5, 64, 1)]
    h = [rng.standard_normal(n).astype(np.float32) for n in (5, 64, 1)]
    r = [0.1, 0.5, 1.0]
    E, Kt = ko.profile(g, h, r)
    assert E.shape == (3, 3) and Kt.tolist() == [[1, 3, 5], [7, 32, 64], [1, 1, 1]]
    for i in range(3):
        x = g[i] - h[i]
        sq = np.sort(x.astype(np.float64) ** 2)
        for j in range(3):
            assert E[i, j] == pytest.approx(math.fsum(sq[: len(x) - Kt[i, j]].tolist()), rel=1e-13, abs=0.0)
