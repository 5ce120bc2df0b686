"""Pins of the oracle's variants: dense fallback of the allocation (reading R15), half-precision payload values
(reading R16), and the baseline allocators of Section 4.3.  None of them compares the oracle with itself: brute
force over all assignments with the byte and error rule written out from its definition, bit patterns worked out
by hand from the binary16 format, invariants the paper states (the plateau at the uncompressed size), and full
sorts of the concatenation."""
import itertools
from fractions import Fraction

import numpy as np

from oracle import kimad_oracle as ko


# ------------------------------------------------------------------ dense fallback
def _send(E_row, K_row, n, j, pair_bytes):
    """bytes and error of layer (row) at grid point j, from the rule itself: pairs, or the bare values if cheaper."""
    K = int(K_row[j])
    if K * pair_bytes >= n * 4:
        return -(-n * 4 // pair_bytes) * pair_bytes, 0.0, n
    return K * pair_bytes, float(E_row[j]), K


def _brute_dense(E, Kt, sizes, budget, pair_bytes):
    L, J = E.shape
    best = None
    for js in itertools.product(range(J), repeat=L):
        total_b, total_e = 0, 0.0
        for i, j in enumerate(js):
            b, e, _ = _send(E[i], Kt[i], sizes[i], j, pair_bytes)
            total_b += b
            total_e = total_e + e                     # left to right, as the programme adds
        if total_b > budget:
            continue
        key = (total_e, total_b, js)                  # least error, then least cost, then lowest j from the last layer back
        if best is None or (total_e, total_b) < best[:2]:
            best = key
    return best


def test_dense_fallback_against_brute_force():
    rng = np.random.default_rng(5)
    for trial in range(40):
        L, J = int(rng.integers(1, 5)), int(rng.integers(2, 5))
        sizes = [int(x) for x in rng.integers(4, 40, size=L)]
        ratios = np.sort(rng.uniform(0.05, 1.0, size=J))
        Kt = np.array([ko.grid_sizes(ratios, n) for n in sizes])
        E = np.sort(rng.integers(1, 50, size=(L, J)).astype(np.float64), axis=1)[:, ::-1].copy()
        E[Kt == np.array(sizes)[:, None]] = 0.0
        budget = int(rng.integers(8, 8 * sum(sizes)))
        st, j, K, off = ko.allocate(E, Kt, budget, 8, 0, dense_sizes=sizes)
        want = _brute_dense(E, Kt, sizes, budget, 8)
        if want is None:
            assert st == ko.ERR_INFEASIBLE
            continue
        assert st == ko.OK
        got_b = sum(_send(E[i], Kt[i], sizes[i], int(j[i]), 8)[0] for i in range(L))
        got_e = 0.0
        for i in range(L):
            got_e = got_e + _send(E[i], Kt[i], sizes[i], int(j[i]), 8)[1]
        assert got_e == want[0] and got_b == want[1], (trial, got_e, got_b, want)
        assert got_b <= budget
        for i in range(L):
            assert int(K[i]) == _send(E[i], Kt[i], sizes[i], int(j[i]), 8)[2]


def test_dense_fallback_plateau_and_dominance():
    """Section 4.2: with bandwidth to spare the sent size levels off at the uncompressed size.  Charged bytes never
    exceed 4 bytes per element; a budget of the bare values sends everything with zero error; the fallback never
    does worse than the plain programme on the same budget."""
    rng = np.random.default_rng(6)
    sizes = [1000, 37, 5000, 64]
    ratios = np.logspace(-2, 0, 12)
    Kt = np.array([ko.grid_sizes(ratios, n) for n in sizes])
    E = np.array([(1.0 - Kt[i] / sizes[i]) ** 2 * rng.uniform(1, 9) for i in range(4)])
    dense_bytes = sum(-(-4 * n // 8) * 8 for n in sizes)
    st, j, K, off = ko.allocate(E, Kt, dense_bytes, 8, 0, dense_sizes=sizes)
    assert st == ko.OK and list(K) == sizes                       # the plateau: everything, at half the pairs' price
    st0, j0, K0, off0 = ko.allocate(E, Kt, dense_bytes, 8, 0)
    assert sum(E[i, j0[i]] for i in range(4)) > 0.0               # the plain programme cannot afford it
    Ev, Kc, Ks = ko.dense_view(E, Kt, sizes, 8)
    assert np.all(Kc * 8 <= -(-4 * np.array(sizes)[:, None] // 8) * 8) and np.all(Kc <= Kt)
    assert np.all(Ev[Kt * 8 >= 4 * np.array(sizes)[:, None]] == 0.0) and np.all((Ks == Kt) | (Ks == np.array(sizes)[:, None]))
    for budget in (800, 4000, 12000, 20000):
        for D in (0, 50):
            a = ko.allocate(E, Kt, budget, 8, D, dense_sizes=sizes)
            b = ko.allocate(E, Kt, budget, 8, D)
            if b[0] == ko.OK:
                assert a[0] == ko.OK
                ea = sum(Ev[i, a[1][i]] for i in range(4))
                eb = sum(E[i, b[1][i]] for i in range(4))
                assert ea <= eb
                assert sum(int(Kc[i, a[1][i]]) for i in range(4)) * 8 <= budget


# ------------------------------------------------------------------ half-precision values
def test_binary16_bit_patterns_by_hand():
    """sign 1 | exponent 5 (bias 15) | fraction 10.  Worked out from the format, not from a library."""
    cases = [
        (1.0, 0x3C00), (-2.0, 0xC000), (0.5, 0x3800), (65504.0, 0x7BFF), (-65504.0, 0xFBFF),
        (70000.0, 0x7BFF), (-1e30, 0xFBFF), (np.inf, 0x7BFF), (-np.inf, 0xFBFF),      # saturated, never infinite
        (2.0 ** -14, 0x0400),                      # smallest normal
        (2.0 ** -24, 0x0001),                      # smallest subnormal
        (2.0 ** -25, 0x0000),                      # halfway to it: ties to even, i.e. to zero
        (2.0 ** -25 * 1.5, 0x0001),                # above halfway
        (1e-8, 0x0000), (-1e-8, 0x8000), (0.0, 0x0000), (-0.0, 0x8000),
        (1.0 + 2.0 ** -11, 0x3C00),                # halfway between 1 and 1 + 2^-10: to the even fraction 0
        (1.0 + 3 * 2.0 ** -11, 0x3C02),            # halfway between fractions 1 and 2: to the even 2
        (1.0 + 2.0 ** -11 + 2.0 ** -20, 0x3C01),   # just above halfway
        (0.1, 0x2E66),                             # 0.1 = 1.6 * 2^-4: exponent 11, fraction round(0.6 * 1024) = 614 = 0x266
    ]
    v = np.array([c[0] for c in cases], dtype=np.float32)
    want = np.array([c[1] for c in cases], dtype=np.uint16)
    assert np.array_equal(ko.quantise_f16(v), want)
    nan = ko.quantise_f16(np.array([np.nan], dtype=np.float32))
    assert (nan[0] & 0x7C00) == 0x7C00 and (nan[0] & 0x03FF) != 0
    # decoding is exact: value = (-1)^s 2^(e-15) (1 + f/1024), or 2^-14 f/1024 for e = 0
    for bits in (0x3C00, 0x2E66, 0x0001, 0x7BFF, 0xC000, 0x03FF):
        s, e, f = bits >> 15, (bits >> 10) & 31, bits & 1023
        val = Fraction(f, 1024) * Fraction(1, 2 ** 14) if e == 0 else (1 + Fraction(f, 1024)) * Fraction(2) ** (e - 15)
        assert Fraction(float(ko.dequantise_f16(np.array([bits], dtype=np.uint16))[0])) == (-val if s else val)


def test_half_precision_payload_keeps_worker_and_server_estimators_equal():
    rng = np.random.default_rng(7)
    g = (rng.standard_normal(300) * 10.0 ** rng.uniform(-6, 5, size=300)).astype(np.float32)
    h = (rng.standard_normal(300) * 0.1).astype(np.float32)
    idx, bits, h_new = ko.compress_ef_layer(g, h, 40, value_format="f16")
    idx32, val32, h_new32 = ko.compress_ef_layer(g, h, 40)
    assert bits.dtype == np.uint16 and np.array_equal(idx, idx32)                 # the support does not depend on the format
    assert np.array_equal(bits, ko.quantise_f16(val32))
    # the server's copy: old h plus the decoded payload, one fp32 addition per pair
    server = h.copy()
    for p in range(len(idx)):
        server[idx[p]] = np.float32(server[idx[p]]) + np.float32(ko.dequantise_f16(bits[p:p + 1])[0])
    assert np.array_equal(server.view(np.uint32), h_new.view(np.uint32))
    hats, _ = ko.server_apply([(np.array([0, 40], dtype=np.uint64), idx, bits)], [h], [1.0], None, 0.0, [0, 300])
    assert np.array_equal(hats[0].view(np.uint32), h_new.view(np.uint32))
    # off the support nothing moved; on it the residual g - h_new is what the rounding lost (or the saturated part)
    off = np.ones(300, dtype=bool); off[idx] = False
    assert np.array_equal(h_new[off].view(np.uint32), h[off].view(np.uint32))
    x = ko.operand(g, h)
    small = np.abs(x[idx]) < 60000
    assert np.all(np.abs((g - h_new)[idx][small]) <= np.abs(x[idx][small]) * 2.0 ** -10 + 2.0 ** -24)


# ------------------------------------------------------------------ baseline allocators
def test_uniform_and_whole_model_sizes():
    rng = np.random.default_rng(8)
    sizes = [50, 7, 300, 1]
    gL = [(rng.standard_normal(n) * s).astype(np.float32) for n, s in zip(sizes, (1.0, 100.0, 0.01, 5.0))]
    hL = [(rng.standard_normal(n) * s).astype(np.float32) for n, s in zip(sizes, (0.5, 300.0, 0.01, 0.0))]
    d = sum(sizes)
    for P in (1, 10, 57, 200, d, d + 50):
        Ku = ko.uniform_sizes(sizes, 8 * P)
        rho = min(1.0, P / d)
        assert list(Ku) == [min(n, max(1, int(np.ceil(rho * n)))) for n in sizes]
        Kw = ko.whole_model_sizes(gL, hL, 8 * P)
        assert Kw.sum() == min(P, d) and np.all(Kw <= np.array(sizes))
        # the definition on the concatenation: a magnitude threshold, everything above it kept
        x = np.concatenate([g - h for g, h in zip(gL, hL)])      # fp32 differences: what is compressed is g - h
        order = np.argsort(-np.abs(x).astype(np.float64), kind="stable")
        kept = np.zeros(d, dtype=bool); kept[order[:min(P, d)]] = True
        pos = 0
        for i, n in enumerate(sizes):
            assert Kw[i] == kept[pos:pos + n].sum()
            pos += n
        # per-layer attribution adds up to the whole model's error, and the whole-model choice is the floor
        Ew = ko.errors_at(gL, hL, Kw)
        whole = np.sort(x[~kept].astype(np.float64) ** 2).sum()
        assert abs(Ew.sum() - whole) <= 1e-12 * max(whole, 1e-300)
        if Ku.sum() <= min(P, d):
            assert Ew.sum() <= ko.errors_at(gL, hL, Ku).sum() * (1 + 1e-12)
    full = ko.errors_at(gL, hL, [0, 0, 0, 0])                     # K = 0: everything is dropped
    for i, (g, h) in enumerate(zip(gL, hL)):
        xi = (g - h).astype(np.float64)
        assert abs(full[i] - float(np.dot(xi, xi))) <= 1e-12 * full[i]
