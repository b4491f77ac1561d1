"""Pins for the oracle's quantisers (Section 3.2.2, Eq.5-7) against what the paper's
formulas and plain mathematics fix: closed forms, invariants, and a literal
evaluation of the printed formulas in exact rational arithmetic."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import quant as oq


# ---- literal formulas, exact rationals (independent of the integer formulation) ----
def R_half_even(fr: Fraction) -> int:
    fl = math.floor(fr)
    d = fr - fl
    if d > Fraction(1, 2) or (d == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def Q_lit(x: Fraction, k=8) -> Fraction:
    return Fraction(R_half_even(x * 2 ** (k - 1)), 2 ** (k - 1))


def CQ_lit(x: Fraction, k=8) -> Fraction:
    b = 1 - Fraction(1, 2 ** (k - 1))
    return max(-b, min(b, Q_lit(x, k)))


def SQ_lit(xs, k=8):
    m = max(abs(x) for x in xs)
    lg = math.log2(float(m))          # Eq.7 as printed; never within 1e-9 of a tie for rationals used here
    assert abs((lg % 1.0) - 0.5) > 1e-9
    scale = Fraction(2) ** round(lg)
    return [scale * CQ_lit(x / scale, k) for x in xs], scale


def test_rne_shift_truth_table():
    v = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, -1, -2, -3, -4, -5, -6, -7, -8, 64, 192, 320, -64, -192, -320])
    # v / 4 -> nearest, ties to even
    want4 = [0, 0, 0, 1, 1, 1, 2, 2, 2, 0, 0, -1, -1, -1, -2, -2, -2, 16, 48, 80, -16, -48, -80]
    assert oq.rne_shift(v, 2).tolist() == want4
    # v / 128: 64 -> 0 (tie to even), 192 -> 2, 320 -> 2 (2.5 -> 2)
    assert oq.rne_shift(np.array([64, 192, 320, -64, -192, -320]), 7).tolist() == [0, 2, 2, 0, -2, -2]
    assert oq.rne_shift(np.array([3, -3]), 0).tolist() == [3, -3]
    assert oq.rne_shift(np.array([3, -3]), -4).tolist() == [48, -48]
    rng = np.random.default_rng(1)
    v = rng.integers(-2 ** 40, 2 ** 40, size=2000)
    for s in (1, 3, 7, 13, 31):
        got = oq.rne_shift(v, s)
        want = [R_half_even(Fraction(int(x), 2 ** s)) for x in v]
        assert got.tolist() == want


def test_q_ties_and_invariants():
    # Eq.5 with ties to even on the 1/128 grid
    x = np.array([0.5 / 128, 1.5 / 128, -2.5 / 128, 2.5 / 128, 0.49 / 128, 300.2 / 128])
    assert oq.q_code(x).tolist() == [0, 2, -2, 2, 0, 300]
    rng = np.random.default_rng(2)
    x = rng.normal(size=5000) * 3
    c = oq.q_code(x)
    assert np.array_equal(oq.q_code(c / 128.0), c)                    # idempotent
    assert np.array_equal(oq.q_code(-x), -c)                          # odd
    assert np.max(np.abs(c / 128.0 - x)) <= 2.0 ** -8 + 1e-15         # half a step
    xs = np.sort(x)
    assert np.all(np.diff(oq.q_code(xs)) >= 0)                        # monotone
    for v in x[:200]:
        assert Fraction(int(oq.q_code(v)), 128) == Q_lit(Fraction(float(v)))


def test_cq_range_and_agreement():
    assert oq.cq_code(np.array([1.0, -1.0, 5.0, -5.0, 127 / 128, -127 / 128])).tolist() == \
        [127, -127, 127, -127, 127, -127]
    rng = np.random.default_rng(3)
    x = rng.uniform(-127 / 128, 127 / 128, size=3000)
    assert np.array_equal(oq.cq_code(x), oq.q_code(x))                # CQ = Q inside the range
    x = rng.normal(size=3000) * 2
    c = oq.cq_code(x)
    assert c.min() >= -127 and c.max() <= 127
    for v in x[:200]:
        assert Fraction(int(oq.cq_code(v)), 128) == CQ_lit(Fraction(float(v)))


def test_scale_exponent_closed_forms():
    # R(log2 M): powers of two, and both sides of sqrt(2)*2^p
    for p in range(0, 40):
        assert oq.scale_exponent_int(1 << p) == p
    assert oq.scale_exponent_int(3) == 2        # log2 3 = 1.585
    assert oq.scale_exponent_int(5) == 2        # 2.32
    assert oq.scale_exponent_int(6) == 3        # 2.585
    assert oq.scale_exponent_int(181) == 7      # 181/128 = 1.4140 < sqrt2
    assert oq.scale_exponent_int(182) == 8      # 1.4219 > sqrt2
    assert oq.scale_exponent_int(300) == 8
    for M in list(range(1, 3000)) + [2 ** 31 - 1, 2 ** 33 + 12345, 46341, 46340]:
        assert oq.scale_exponent_int(M) == round(math.log2(M)), M
    assert oq.scale_exponent_real(0.3) == -2
    assert oq.scale_exponent_real(1.0) == 0
    assert oq.scale_exponent_real(1.41) == 0
    assert oq.scale_exponent_real(1.42) == 1
    assert oq.scale_exponent_real(2.0 ** -30) == -30
    rng = np.random.default_rng(4)
    for v in np.exp(rng.uniform(-30, 30, size=2000)):
        assert oq.scale_exponent_real(v) == round(math.log2(v))


def test_sq_hand_examples():
    # x = {0.3, -0.1}: log2 0.3 = -1.737 -> R = -2, scale 1/4; x/scale*128 = {153.6, -51.2}
    c, E = oq.sq_real(np.array([0.3, -0.1]))
    assert c.tolist() == [127, -51] and E == -9        # values 127/512, -51/512
    # integers: v = {300, -100} at 2^-20: r = 8, shift 1: {150 -> 127, -50}, E = -19
    c, E = oq.sq_int(np.array([300, -100]), -20)
    assert c.tolist() == [127, -50] and E == -19
    # all-zero tensors keep their exponent / get 0
    c, E = oq.sq_int(np.zeros(4, dtype=np.int64), -11)
    assert c.tolist() == [0, 0, 0, 0] and E == -11
    c, E = oq.sq_real(np.zeros(3))
    assert c.tolist() == [0, 0, 0] and E == 0


def test_sq_matches_literal_formula():
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(1, 12))
        E = int(rng.integers(-30, 5))
        v = rng.integers(-2 ** int(rng.integers(1, 30)), 2 ** int(rng.integers(1, 30)), size=n)
        if not np.any(v):
            continue
        xs = [Fraction(int(a)) * Fraction(2) ** E for a in v]
        lit, scale = SQ_lit(xs)
        c, Eo = oq.sq_int(v, E)
        assert Fraction(2) ** Eo * 128 == scale
        assert [Fraction(int(a)) * Fraction(2) ** Eo for a in c] == lit
        # the real-input path on the same values (exactly representable doubles)
        c2, E2 = oq.sq_real(np.array([float(x) for x in xs]))
        assert E2 == Eo and c2.tolist() == c.tolist()


def test_sq_invariants():
    rng = np.random.default_rng(6)
    for trial in range(50):
        v = rng.integers(-10 ** 6, 10 ** 6, size=500)
        c, E = oq.sq_int(v, -9)
        mx = int(np.abs(c).max())
        assert 91 <= mx <= 127                              # max|x|/scale in (2^-1/2, 2^1/2), clamped
        r = E + 7 - (-9)
        ratio = np.abs(v).max() / 2.0 ** r
        assert 2 ** -0.5 < ratio < 2 ** 0.5
        c2, E2 = oq.sq_int(-v, -9)
        assert np.array_equal(c2, -c) and E2 == E           # odd
        c3, E3 = oq.sq_int(v * 8, -9)
        assert np.array_equal(c3, c) and E3 == E + 3        # SQ(2^j x) = 2^j SQ(x)
        c4, E4 = oq.sq_int(v, -3)
        assert np.array_equal(c4, c) and E4 == E + 6
        c5, E5 = oq.sq_int(c, E)
        assert np.array_equal(c5, c) and E5 == E            # idempotent
        assert np.all(np.sign(c) * np.sign(v) >= 0)


@pytest.mark.parametrize("x,code", [(1.0, 128), (0.0, 0), (-1.0, -128), (1.00390625, 128), (1.01171875, 130)])
def test_scalar_codes_unclamped(x, code):
    # Eq.10: multiplier and bias use the basic quantiser, so 1.0 is code 128
    assert int(oq.q_code(x)) == code
