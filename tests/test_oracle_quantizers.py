"""Pins of the oracle's tables and block quantizers against things other than itself:
exact rational arithmetic, closed forms, hand-derived fixtures, invariants."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")
BITS = [2, 3, 4, 5, 6, 7, 8]


def f32_bits(x):
    return int(np.float32(x).view(np.uint32))


def frac(x):
    return Fraction(float(x))  # exact: every fp32 is a dyadic rational


# ------------------------------------------------------------------ table G
def test_G_powers_of_two_are_exact(oracle):
    for k in range(0, 16):
        assert frac(oracle.G(32 * k)) == Fraction(1, 2 ** k)


def test_G_sqrt_half_bit_pattern(oracle):
    # 2^(-1/2) = 0.70710678118... whose nearest binary32 is 0x3F3504F3 (textbook constant)
    assert f32_bits(oracle.G(16)) == 0x3F3504F3


def test_G_is_nearest_fp32_of_the_exact_root(oracle):
    # G[j]^32 must bracket 2^-j: pred(G)^32 < 2^-j < succ(G)^32, and G is the nearer one.
    for j in range(1, 511):
        g = np.float32(oracle.G(j))
        lo = np.nextafter(g, np.float32(0))
        hi = np.nextafter(g, np.float32(2))
        target = Fraction(1, 2 ** j)
        # midpoints between neighbours: exact value must lie within (mid_lo, mid_hi)
        mid_lo = (frac(lo) + frac(g)) / 2
        mid_hi = (frac(hi) + frac(g)) / 2
        assert mid_lo ** 32 <= target <= mid_hi ** 32, j


def test_G_strictly_decreasing(oracle):
    g = [float(oracle.G(j)) for j in range(511)]
    assert all(a > b for a, b in zip(g, g[1:]))


# ------------------------------------------------------------------ table R
@pytest.mark.parametrize("b", BITS)
def test_R_is_correctly_rounded_quotient(oracle, b):
    qmax = 2 ** (b - 1) - 1
    for u in range(0, 2 * qmax + 1):
        r = np.float32(oracle.R(b, u))
        exact = Fraction(u - qmax, qmax)
        lo = np.nextafter(r, np.float32(-2))
        hi = np.nextafter(r, np.float32(2))
        assert abs(frac(r) - exact) <= abs(frac(lo) - exact)
        assert abs(frac(r) - exact) <= abs(frac(hi) - exact)
    assert oracle.R(b, qmax) == 0.0
    assert oracle.R(b, 0) == -1.0 and oracle.R(b, 2 * qmax) == 1.0


def test_R_2bit_grid(oracle):
    assert [float(oracle.R(2, u)) for u in range(3)] == [-1.0, 0.0, 1.0]


# --------------------------------------------------------------- tables L, T
@pytest.mark.parametrize("b", BITS)
def test_log_levels_and_thresholds(oracle, b):
    kmax = 2 ** b - 1
    step_oct = Fraction(2 ** 4, 2 ** b)  # 2^(4-b) octaves between levels
    assert oracle.Lv(b, kmax) == 1.0  # top code is the block maximum itself
    for c in range(kmax + 1):
        k = kmax - c
        # level = 2^(-k*step): check lv^32 against 2^(-32*k*step) with a 1-ulp bracket
        e = 32 * k * step_oct
        assert e.denominator == 1
        lv = np.float32(oracle.Lv(b, c))
        assert frac(np.nextafter(lv, np.float32(0))) ** 32 < Fraction(1, 2 ** int(e)) < frac(np.nextafter(lv, np.float32(2))) ** 32
    for k in range(kmax):
        # threshold k is the geometric midpoint of levels k and k+1: T^2 ~ L_k * L_{k+1}
        t = float(oracle.T(b, k))
        prod = float(oracle.Lv(b, kmax - k)) * float(oracle.Lv(b, kmax - k - 1))
        assert abs(t * t - prod) <= 4e-7 * prod
        assert oracle.Lv(b, kmax - k) > oracle.T(b, k) > oracle.Lv(b, kmax - k - 1)


def test_log_2bit_levels_are_the_hand_values(oracle):
    assert [float(oracle.Lv(2, c)) for c in (3, 2, 1, 0)] == [1.0, 2.0 ** -4, 2.0 ** -8, 2.0 ** -12]
    assert [float(oracle.T(2, k)) for k in range(3)] == [2.0 ** -2, 2.0 ** -6, 2.0 ** -10]
    assert [float(oracle.Lv(3, c)) for c in range(7, -1, -1)] == [2.0 ** (-2 * k) for k in range(8)]
    assert [float(oracle.Lv(4, c)) for c in range(15, -1, -1)] == [2.0 ** -k for k in range(16)]


@pytest.mark.parametrize("b", BITS[:-1])
def test_log_grids_are_nested(oracle, b):
    fine = {f32_bits(oracle.Lv(b + 1, c)) for c in range(2 ** (b + 1))}
    # the coarse grid reaches further down than the fine one only below the fine grid's floor
    floor = float(oracle.Lv(b + 1, 0))
    for c in range(2 ** b):
        lv = oracle.Lv(b, c)
        if float(lv) >= floor:
            assert f32_bits(lv) in fine


# ------------------------------------------------------------ linear quantizer
def brute_linear(x, b):
    """argmin over the integer grid in exact rational arithmetic; None where tied."""
    qmax = 2 ** (b - 1) - 1
    s = max(abs(frac(v)) for v in x)
    out = []
    for v in x:
        if s == 0:
            out.append(qmax)
            continue
        t = frac(v) / s * qmax
        best = sorted(range(-qmax, qmax + 1), key=lambda q: abs(t - q))
        tied = abs(abs(t - best[0]) - abs(t - best[1])) < Fraction(1, 2 ** 18)
        out.append(None if tied else best[0] + qmax)
    return out


@pytest.mark.parametrize("b", BITS)
def test_linear_matches_exact_nearest_grid_point(oracle, b):
    rng = np.random.default_rng(100 + b)
    for trial in range(40):
        n = int(rng.integers(1, 9))
        x = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 3)).astype(np.float32)
        u, s = oracle.quant_linear_block(x, b)
        assert frac(s) == max(abs(frac(v)) for v in x)
        want = brute_linear(x, b)
        for got, w in zip(u, want):
            if w is not None:  # within 2^-18 of a tie fp32 rounding may pick either side
                assert int(got) == w


@pytest.mark.parametrize("b", BITS)
def test_linear_invariants(oracle, b):
    rng = np.random.default_rng(200 + b)
    qmax = 2 ** (b - 1) - 1
    for K in (1, 7, 64, 128, 256):
        x = (rng.standard_normal(K) * 3e-4).astype(np.float32)
        u, s = oracle.quant_linear_block(x, b)
        assert u.max() <= 2 * qmax  # top code 2^b-1 never used
        imax = int(np.argmax(np.abs(x)))
        assert abs(int(u[imax]) - qmax) == qmax
        y = oracle.dequant_linear_block(u, b, s)
        assert y[imax] == x[imax]  # absmax element is reproduced exactly
        assert np.abs(y).max() == s
        # error bound: half a grid step plus rounding slack
        assert np.all(np.abs(y.astype(np.float64) - x) <= float(s) / (2 * qmax) * (1 + 1e-5))
        # idempotence
        u2, s2 = oracle.quant_linear_block(y, b)
        assert s2 == s and np.array_equal(u2, u)


def test_linear_2bit_exhaustive(oracle):
    # grid {-s, 0, +s}; |x| > s/2 goes to +-s, |x| < s/2 goes to 0, exactly s/2 goes to even (0)
    vals = [-1.0, -0.75, -0.5, -0.25, 0.0, 0.25, 0.5, 0.75, 1.0]
    want = {-1.0: 0, -0.75: 0, -0.5: 1, -0.25: 1, 0.0: 1, 0.25: 1, 0.5: 1, 0.75: 2, 1.0: 2}
    import itertools
    for combo in itertools.product(vals, repeat=3):
        x = np.array((1.0,) + combo, np.float32) * np.float32(0.125)  # element 0 pins the scale
        u, s = oracle.quant_linear_block(x, 2)
        assert s == np.float32(0.125)
        assert [int(t) for t in u] == [2] + [want[c] for c in combo]


def test_linear_half_to_even(oracle):
    # b=4: qmax=7; x/s*7 = 2.5 -> 2, 3.5 -> 4 (ties to even)
    x = np.array([7.0, 2.5, 3.5, -2.5, -3.5], np.float32)
    u, s = oracle.quant_linear_block(x, 4)
    assert s == 7.0 and [int(t) - 7 for t in u] == [7, 2, 4, -2, -4]


def test_linear_outlier_stays_local(oracle):
    # Sec. 3.5: block-wise scales keep an outlier from distorting other blocks
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(256) * 1e-3).astype(np.float32)
    u0, s0 = oracle.quant_linear_block(x[:128], 8)
    x2 = x.copy()
    x2[200] = 50.0
    u1, s1 = oracle.quant_linear_block(x2[:128], 8)
    assert s0 == s1 and np.array_equal(u0, u1)
    _, s_hi = oracle.quant_linear_block(x2[128:], 8)
    assert s_hi == 50.0


def test_zero_and_tiny_blocks(oracle):
    for b in BITS:
        qmax = 2 ** (b - 1) - 1
        u, s = oracle.quant_linear_block(np.zeros(5, np.float32), b)
        assert s == 0 and np.all(u == qmax)
        c, s = oracle.quant_log_block(np.zeros(5, np.float32), b)
        assert s == 0 and np.all(c == 0)
        tiny = np.array([1e-39, -5e-40, 0.0], np.float32)  # below the smallest normal
        u, s = oracle.quant_linear_block(tiny, b)
        assert s == 0 and np.all(u == qmax)
        c, s = oracle.quant_log_block(np.abs(tiny), b)
        assert s == 0 and np.all(c == 0)
        ok = np.array([1.2e-38, 6e-39], np.float32)  # max is normal: handled normally
        u, s = oracle.quant_linear_block(ok, b)
        assert s == ok[0] and u[0] == 2 * qmax


# --------------------------------------------------------------- log quantizer
def parse_pow(tok):
    return 0.0 if tok == "z" else 2.0 ** int(tok)


def test_log_2bit_hand_cases(oracle):
    n = 0
    for line in open(os.path.join(GOLD, "log_2bit_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        lhs, rhs = line.split("->")
        sc, codes = rhs.split(";")
        x = np.array([parse_pow(t) for t in lhs.split()], np.float32)
        c, s = oracle.quant_log_block(x, 2)
        assert float(s) == parse_pow(sc.strip())
        assert [int(t) for t in c] == [int(t) for t in codes.split()], line
        n += 1
    assert n == 8


def test_log_2bit_exhaustive_K4(oracle):
    # all 4^4 code patterns: a block made of level values must quantize back to its own codes
    lv = {3: 1.0, 2: 2.0 ** -4, 1: 2.0 ** -8, 0: 2.0 ** -12}
    import itertools
    for codes in itertools.product(range(4), repeat=4):
        if 3 not in codes:
            continue  # a block always contains its maximum (code 3)
        x = np.array([lv[c] * 2.0 ** -9 for c in codes], np.float32)
        c, s = oracle.quant_log_block(x, 2)
        assert float(s) == 2.0 ** -9 and tuple(int(t) for t in c) == codes


def exact_log_code(rho: Fraction, b: int):
    """code from exact arithmetic: k = #{k' : rho < 2^(-(2k'+1)*2^(3-b))}; rho^32 vs 2^-j is exact."""
    kmax = 2 ** b - 1
    k = 0
    r32 = rho ** 32
    while k < kmax and r32 < Fraction(1, 2 ** ((2 * k + 1) * 2 ** (8 - b))):
        k += 1
    return kmax - k


@pytest.mark.parametrize("b", BITS)
def test_log_matches_exact_thresholds(oracle, b):
    rng = np.random.default_rng(300 + b)
    kmax = 2 ** b - 1
    thr_bits = {f32_bits(oracle.T(b, k)) for k in range(kmax)}
    for trial in range(12):
        n = 16
        x = (2.0 ** rng.uniform(-18, 0, n)).astype(np.float32)
        x[0] = 1.0  # scale 1 -> rho = x exactly
        c, s = oracle.quant_log_block(x, b)
        assert s == 1.0
        for xi, ci in zip(x, c):
            if f32_bits(xi) in thr_bits:
                continue  # equality with the rounded threshold is decided by the tie rule
            assert int(ci) == exact_log_code(frac(xi), b)


@pytest.mark.parametrize("b", BITS)
def test_log_invariants(oracle, b):
    rng = np.random.default_rng(400 + b)
    kmax = 2 ** b - 1
    half_step = 2.0 ** (2.0 ** (4 - b) / 2)
    for K in (1, 5, 64, 128, 256):
        g = rng.standard_normal(K) * 1e-3
        x = (g * g).astype(np.float32)
        c, s = oracle.quant_log_block(x, b)
        imax = int(np.argmax(x))
        assert s == x[imax] and c[imax] == kmax
        y = oracle.dequant_log_block(c, b, s)
        assert y[imax] == x[imax] and y.max() == s and y.min() > 0
        floor = float(s) * float(oracle.Lv(b, 0))
        inside = x >= floor
        ratio = y[inside].astype(np.float64) / x[inside]
        assert np.all(ratio <= half_step * (1 + 1e-6)) and np.all(ratio >= 1 / half_step * (1 - 1e-6))
        assert np.all(y[~inside] == np.float32(floor))  # clamp to the bottom level, never to zero
        c2, s2 = oracle.quant_log_block(y, b)
        assert s2 == s and np.array_equal(c2, c)
        # monotone: larger value never gets a smaller code
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(c[order].astype(int)) >= 0)


def test_log_tie_goes_to_larger_level(oracle):
    for b in BITS:
        kmax = 2 ** b - 1
        for k in (0, kmax // 2, kmax - 1):
            t = oracle.T(b, k)
            x = np.array([1.0, t, np.nextafter(t, np.float32(0))], np.float32)
            c, _ = oracle.quant_log_block(x, b)
            assert int(c[1]) == kmax - k and int(c[2]) == kmax - k - 1
