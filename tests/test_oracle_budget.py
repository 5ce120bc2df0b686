"""Pins of the oracle's budget rule (Section 3.1, Eq. budget) against what the paper fixes:
the printed formula at alpha = 1, the time split it is derived from, and the experiment's
shortcut c = T_comm * B (Section 4.2, Setting)."""
from fractions import Fraction

import numpy as np

from oracle import kimad_oracle as ko


def test_alpha_one_is_the_printed_formula():
    # exact rational arithmetic on values that are exact in binary
    for B, t, tc in [(2 ** 30, 0.5, 0.25), (3 * 2 ** 20, 1.0, 0.125), (10 ** 9, 0.75, 0.5)]:
        want = Fraction(B) * (Fraction(t) - Fraction(tc)) / 2 / 8
        assert ko.budget_bytes(B, t, tc) == want.numerator // want.denominator


def test_budget_fills_the_time_split_exactly():
    """t = c/B + T_comp + alpha c/B must hold for the c behind the returned bytes (up to the byte floor)."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        B = float(rng.uniform(30e6, 330e6))          # the paper's 30..330 Mbps
        tc = float(rng.uniform(0.0, 0.2))
        t = tc + float(rng.uniform(1e-3, 1.0))
        alpha = float(rng.choice([0.0, 0.5, 1.0, 2.0]))
        nbytes = ko.budget_bytes(B, t, tc, alpha)
        c_lo, c_hi = 8.0 * nbytes, 8.0 * (nbytes + 1)
        t_lo = c_lo / B + tc + alpha * c_lo / B
        t_hi = c_hi / B + tc + alpha * c_hi / B
        assert t_lo <= t * (1 + 1e-12) and t < t_hi * (1 + 1e-12)


def test_experiment_shortcut_and_degenerate_cases():
    # Section 4.2: with alpha = 1 the budget is T_comm * B, T_comm the time of one direction
    B, t_comm, tc = 100e6, 0.05, 0.01
    assert ko.budget_bytes(B, 2 * t_comm + tc, tc) == int(np.floor(t_comm * B / 8))
    assert ko.budget_bytes(B, tc, tc) == 0 and ko.budget_bytes(B, 0.0, tc) == 0
    assert ko.budget_bytes(0.0, 1.0, 0.0) == 0 and ko.budget_bytes(float("nan"), 1.0, 0.0) == 0
    assert ko.budget_bytes(B, 1.0, 0.0, cap_bytes=1000) == 1000
    # a one-directional link (alpha = 0) gets the whole communication time
    assert ko.budget_bytes(B, 1.0, 0.5, alpha=0.0) == int(np.floor(B * 0.5 / 8))
