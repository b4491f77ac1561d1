"""Oracle: the three quantisers of Section 3.2.2 and their per-data strategies
(Section 3.2.3).  TEST INFRASTRUCTURE ONLY -- see the package docstring.

Bit width k = 8 everywhere (Section 5.1).  A quantised value is an integer
*code* times a power of two:
    Q(x, 8)  <-> code = R(128 x)                     value = code / 128
    CQ(x, 8) <-> code = clamp(R(128 x), -127, 127)   (bounds +-(1 - 2^-7))
    SQ(x, 8) <-> scale = 2^R(log2 max|x|), code = CQ(x / scale), value = code * scale / 128
R() rounds to nearest, ties to even (the paper leaves the tie rule open).
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

K_BITS = 8
ONE = 1 << (K_BITS - 1)        # 128: codes per unit
CODE_MAX = ONE - 1             # 127


# --------------------------------------------------------------------------
# rounding
# --------------------------------------------------------------------------
def rne_shift(v, s: int):
    """v * 2^-s rounded to the nearest integer, ties to even (s >= 1); exact
    left shift for s <= 0.  Written as the plain definition: floor quotient,
    remainder, compare with one half."""
    v = np.asarray(v, dtype=np.int64)
    if s <= 0:
        return v * (np.int64(1) << np.int64(-s))
    s = min(int(s), 62)                         # |v| < 2^61 here: larger shifts all give 0
    q = v >> np.int64(s)                        # floor(v / 2^s)
    rem = v - (q << np.int64(s))                # in [0, 2^s)
    half = np.int64(1) << np.int64(s - 1)
    up = (rem > half) | ((rem == half) & ((q & 1) == 1))
    return q + up.astype(np.int64)


# --------------------------------------------------------------------------
# real-valued inputs (network input, head error, initial weights)
# --------------------------------------------------------------------------
def q_code(x) -> np.ndarray:
    """Eq.5 (basic quantiser): integer code R(x * 2^(k-1)); unbounded."""
    x = np.asarray(x, dtype=np.float64)
    return np.rint(x * float(ONE)).astype(np.int64)


def cq_code(x) -> np.ndarray:
    """Eq.6 (clamp quantiser): Eq.5 then clamp to +-(1 - 2^-(k-1)), i.e. codes +-127."""
    return np.clip(q_code(x), -CODE_MAX, CODE_MAX)


def scale_exponent_real(maxabs: float) -> int:
    """R(log2(maxabs)) of Eq.7 for a positive finite float, without calling log:
    maxabs = f * 2^e with f in [1/2, 1); log2 f >= -1/2  <=>  f^2 >= 1/2, and
    equality is impossible for a rational f, so there is never a tie."""
    f, e = math.frexp(float(maxabs))
    return e if Fraction(f) ** 2 > Fraction(1, 2) else e - 1


def sq_real(x):
    """Eq.7 on real input: returns (int codes, E) with value = code * 2^E.
    scale = 2^R; x / scale * 128 = x * 2^(7-R); E = R - 7.  All-zero input:
    codes 0, E = 0 (the paper does not define log2 0)."""
    x = np.asarray(x, dtype=np.float64)
    m = float(np.max(np.abs(x))) if x.size else 0.0
    if m == 0.0:
        return np.zeros(x.shape, dtype=np.int64), 0
    R = scale_exponent_real(m)
    scaled = np.ldexp(x, (K_BITS - 1) - R)      # exact: power-of-two factor
    codes = np.clip(np.rint(scaled).astype(np.int64), -CODE_MAX, CODE_MAX)
    return codes, R - (K_BITS - 1)


# --------------------------------------------------------------------------
# integer inputs: v * 2^E with integer v (everything in the backward pass)
# --------------------------------------------------------------------------
def scale_exponent_int(M: int) -> int:
    """R(log2 M) for an integer M >= 1: p = floor(log2 M); round up iff
    log2 M - p > 1/2  <=>  M^2 > 2^(2p+1)  (never equal for an integer)."""
    M = int(M)
    p = M.bit_length() - 1
    return p + (1 if M * M > (1 << (2 * p + 1)) else 0)


def sq_int(v, E: int):
    """Eq.7 on v * 2^E: scale = 2^(E + r), r = R(log2 max|v|);
    code = CQ(v * 2^E / scale) = clamp(R(v * 2^(7-r))); value = code * 2^(E + r - 7).
    All-zero input: codes 0, exponent unchanged."""
    v = np.asarray(v, dtype=np.int64)
    M = int(np.max(np.abs(v))) if v.size else 0
    if M == 0:
        return np.zeros(v.shape, dtype=np.int64), int(E)
    r = scale_exponent_int(M)
    codes = np.clip(rne_shift(v, r - (K_BITS - 1)), -CODE_MAX, CODE_MAX)
    return codes, int(E) + r - (K_BITS - 1)
