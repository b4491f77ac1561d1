"""Oracle: one Fixup layer forward (Eq.2), backward (Eq.3), parameter gradients
(Eq.4) and the 8-bit update (Eq.13), on integer codes.
TEST INFRASTRUCTURE ONLY -- see the package docstring.

Grids: int8 activations, weights and the scalar codes (bias, multiplier) sit on
2^-7; a conv accumulator sits on 2^-14.  Backward tensors are (int8 codes, E)
with value = code * 2^E.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass

import numpy as np

from . import build as _build
from .quant import CODE_MAX, ONE, rne_shift, sq_int

_lib = None


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "K", "R", "S", "stride", "pad")]


@dataclass(frozen=True)
class ConvShape:
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def c(self):
        return _Desc(self.N, self.H, self.W, self.C, self.K, self.R, self.S, self.stride, self.pad)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        for f in ("eo_conv_fwd", "eo_conv_bwd_data", "eo_conv_bwd_weight"):
            getattr(_lib, f).restype = C.c_long
        _lib.eo_head_exp.restype = C.c_double
        _lib.eo_head_exp.argtypes = [C.c_double]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int8, a.dtype
    return a


# --------------------------------------------------------------------------
# convolutions (direct loops in C)
# --------------------------------------------------------------------------
def conv_fwd(d: ConvShape, u, w) -> np.ndarray:
    u, w = _i8(u), _i8(w)
    assert u.shape == (d.N, d.H, d.W, d.C) and w.shape == (d.K, d.R, d.S, d.C)
    acc = np.empty((d.N, d.P, d.Q, d.K), dtype=np.int32)
    bad = lib().eo_conv_fwd(C.byref(d.c()), _p(u), _p(w), _p(acc))
    assert bad == 0, "forward accumulator left int32"
    return acc


def conv_bwd_data(d: ConvShape, e, w) -> np.ndarray:
    e, w = _i8(e), _i8(w)
    assert e.shape == (d.N, d.P, d.Q, d.K) and w.shape == (d.K, d.R, d.S, d.C)
    dx = np.empty((d.N, d.H, d.W, d.C), dtype=np.int32)
    bad = lib().eo_conv_bwd_data(C.byref(d.c()), _p(e), _p(w), _p(dx))
    assert bad == 0, "backward-data accumulator left int32"
    return dx


def conv_bwd_weight(d: ConvShape, e, u) -> np.ndarray:
    e, u = _i8(e), _i8(u)
    assert e.shape == (d.N, d.P, d.Q, d.K) and u.shape == (d.N, d.H, d.W, d.C)
    g = np.empty((d.K, d.R, d.S, d.C), dtype=np.int32)
    bad = lib().eo_conv_bwd_weight(C.byref(d.c()), _p(e), _p(u), _p(g))
    assert bad == 0, "weight-gradient accumulator left int32"
    return g


def maxpool_fwd(a, R=3, S=3, stride=2, pad=1):
    a = _i8(a)
    N, H, W, Cc = a.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.empty((N, P, Q, Cc), dtype=np.int8)
    arg = np.empty((N, P, Q, Cc), dtype=np.uint8)
    lib().eo_maxpool_fwd(N, H, W, Cc, R, S, stride, pad, _p(a), _p(y), _p(arg))
    return y, arg


def maxpool_bwd(e, arg, in_shape, R=3, S=3, stride=2, pad=1):
    e = _i8(e)
    N, H, W, Cc = in_shape
    d = np.empty(in_shape, dtype=np.int32)
    lib().eo_maxpool_bwd(N, H, W, Cc, R, S, stride, pad, _p(e), _p(np.ascontiguousarray(arg)), _p(d))
    return d


def head(gap_sum, Wfc, bfc, labels, HW):
    """Float head (see eoq_oracle.c): returns loss, d (fp32 error per real
    activation, [N,F]), dW, db, logits."""
    gap_sum = np.ascontiguousarray(gap_sum, dtype=np.int32)
    Wfc = np.ascontiguousarray(Wfc, dtype=np.float64)
    bfc = np.ascontiguousarray(bfc, dtype=np.float64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    N, F = gap_sum.shape
    J = Wfc.shape[0]
    loss = C.c_double(0.0)
    d = np.empty((N, F), dtype=np.float32)
    dW = np.empty((J, F), dtype=np.float64)
    db = np.empty((J,), dtype=np.float64)
    logits = np.empty((N, J), dtype=np.float64)
    lib().eo_head(N, F, J, HW, _p(gap_sum), _p(Wfc), _p(bfc), _p(labels), C.byref(loss), _p(d), _p(dW),
                  _p(db), _p(logits))
    return loss.value, d, dW, db, logits


# --------------------------------------------------------------------------
# one Fixup layer, forward (Eq.2)
# --------------------------------------------------------------------------
def pre_bias(a, b_pre: int) -> np.ndarray:
    """x1 = x0 + Q_b(b1), saturated to the int8 code range so that it can feed
    an int8 convolution (identity at the initial value b = 0)."""
    return np.clip(a.astype(np.int64) + int(b_pre), -CODE_MAX, CODE_MAX).astype(np.int8)


def q_a1(acc) -> np.ndarray:
    """x2 = Q_a1(conv): basic quantiser (Eq.9), grid 2^-14 -> 2^-7, not clamped."""
    return rne_shift(acc, 7)


def post_conv(t, gamma: int, b_post: int, skip=None) -> np.ndarray:
    """x4 on the 2^-14 grid: gamma*x2 + b2 (+ the residual input of the block)."""
    z = int(gamma) * t.astype(np.int64) + ONE * int(b_post)
    if skip is not None:
        z = z + ONE * skip.astype(np.int64)
    return z


def relu_q_a2(z):
    """x5 = Q_a2(relu(x4)): clamp quantiser (Eq.9) -> int8 codes in [0,127];
    mask = relu'(x4) = [x4 > 0] on the unquantised value (straight-through
    estimator, Section 3.2)."""
    y = np.clip(rne_shift(np.maximum(z, 0), 7), 0, CODE_MAX).astype(np.int8)
    return y, (z > 0)


# --------------------------------------------------------------------------
# backward pieces (Eq.3, Eq.4)
# --------------------------------------------------------------------------
def sq_error_gamma(e1, E: int, gamma: int):
    """e3 = Q_e(e2 * Q_gamma(gamma)): product on grid 2^(E-7), then SQ."""
    codes, E3 = sq_int(e1.astype(np.int64) * int(gamma), E - 7)
    return codes.astype(np.int8), E3


def sq_acc(acc, E: int):
    """SQ of an int32 accumulator tensor acc * 2^E -> (int8, E')."""
    codes, Eo = sq_int(acc, E)
    return codes.astype(np.int8), Eo


def merge_errors(ea, Ea: int, eb, Eb: int, max_gap: int = 24):
    """Error entering a block = branch error + shortcut error (both int8 with
    their own exponents): aligned exactly on the finer grid, added, then Q_e."""
    Em = min(Ea, Eb)
    assert max(Ea, Eb) - Em <= max_gap, "exponent gap too large"
    v = ea.astype(np.int64) * (1 << (Ea - Em)) + eb.astype(np.int64) * (1 << (Eb - Em))
    codes, Eo = sq_int(v, Em)
    return codes.astype(np.int8), Eo


def scalar_gradient(terms, max_gap: int = 24):
    """Gradient of a scalar parameter (Eq.4): the sum over all elements, then
    Q_g of the one-element tensor.  `terms` = [(S, E), ...] integer sums with
    their exponents (two terms when two convolutions share the biased input)."""
    Em = min(E for _, E in terms)
    tot = 0
    for S, E in terms:
        assert E - Em <= max_gap
        tot += int(S) << (E - Em)
    codes, Eg = sq_int(np.array([tot], dtype=np.int64), Em)
    return int(codes[0]), Eg


# --------------------------------------------------------------------------
# update (Eq.13) with lr = m * 2^-j
# --------------------------------------------------------------------------
# ---- optional stochastic rounding of the update (NOT in the paper; off unless asked for) --------------------
# With round-to-nearest an update below half a code vanishes, so at small learning rates the 8-bit weights never
# move.  The optional mode rounds u_code * 2^(Eu+7) to one of its two neighbours with probabilities proportional to
# the distance from the other (unbiased): d = floor((u_code + r) / 2^s), r uniform in [0, 2^s), s = -(Eu + 7) > 0
# (an exact left shift otherwise).  r is the low s bits (s capped at 62) of a counter-based 64-bit hash of
# (seed, tensor id, step, element index), so that every element's draw can be regenerated on its own:
#     z = seed*A + tensor*B + step*C + index*D  (mod 2^64),  word = finalise(z)   (the splitmix64 finaliser)
SR_A, SR_B, SR_C, SR_D = 0x9E3779B97F4A7C15, 0xC2B2AE3D27D4EB4F, 0xA0761D6478BD642F, 0xD6E8FEB86659FD93
_M64 = (1 << 64) - 1


def sr_words(seed: int, tensor: int, step: int, n: int) -> np.ndarray:
    """64-bit hash words for elements 0 .. n-1 of one tensor in one step (uint64)."""
    base = (int(seed) * SR_A + int(tensor) * SR_B + int(step) * SR_C) & _M64
    with np.errstate(over="ignore"):
        z = np.arange(n, dtype=np.uint64) * np.uint64(SR_D) + np.uint64(base)
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return z


def sr_shift(v, s: int, words) -> np.ndarray:
    """v * 2^-s rounded stochastically with the given hash words (one per element); exact left shift for s <= 0."""
    v = np.asarray(v, dtype=np.int64)
    if s <= 0:
        return v * (np.int64(1) << np.int64(-s))
    s = min(int(s), 62)
    r = (np.asarray(words, dtype=np.uint64) & np.uint64((1 << s) - 1)).astype(np.int64)
    return (v + r) >> np.int64(s)               # arithmetic shift = floor, also for negative sums


def update_delta(g_codes, Eg: int, lr_m: int, lr_j: int, sr=None) -> np.ndarray:
    """Q_u(lr*g) re-expressed on the parameter grid 2^-7:
    u = SQ(m*g * 2^(Eg-j)) -> (u_code, Eu); delta = R(u_code * 2^(Eu+7)).
    sr = (seed, tensor id, step): the optional stochastic rounding above instead of R."""
    u, Eu = sq_int(np.asarray(g_codes, dtype=np.int64) * int(lr_m), Eg - int(lr_j))
    if sr is None:
        return rne_shift(u, -(Eu + 7))
    seed, tensor, step = sr
    return sr_shift(u, -(Eu + 7), sr_words(seed, tensor, step, u.size).reshape(u.shape))


def update_weights(W, g_codes, Eg, lr_m, lr_j, sr=None) -> np.ndarray:
    """W <- Q_w(W - Q_u(lr*g)) = clamp(W - delta, -127, 127) on int8 codes."""
    d = update_delta(g_codes, Eg, lr_m, lr_j, sr)
    return np.clip(W.astype(np.int64) - d, -CODE_MAX, CODE_MAX).astype(np.int8)


def update_scalar(code: int, g_code: int, Eg: int, lr_m: int, lr_j: int, sr=None) -> int:
    """Bias / multiplier codes use the unclamped basic quantiser (Eq.10)."""
    d = update_delta(np.array([g_code]), Eg, lr_m, lr_j, sr)
    new = int(code) - int(d[0])
    assert -2 ** 31 < new < 2 ** 31, "scalar code left the int32 range it is stored in"
    return new
