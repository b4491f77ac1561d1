"""Pins for the oracle's layer arithmetic: Eq.2 evaluated literally in real numbers,
epilogue special cases, the 8-bit update (Eq.13), Fixup initialisation (Eq.1), the pool
and the float head."""
import math

import numpy as np
import pytest

import seeded_inputs as si
from oracle import fixup, ops
from oracle import quant as oq
from oracle.ops import ConvShape


def test_layer_forward_equals_literal_real_formulas():
    # Eq.2 in doubles (all values are dyadic rationals far inside 53 bits, so this is exact)
    d = ConvShape(2, 6, 6, 8, 8, 3, 3, 1, 1)
    a = si.uniform_int8(0, "a", (d.N, d.H, d.W, d.C))
    w = si.uniform_int8(0, "w", (d.K, d.R, d.S, d.C), -40, 40)
    for b1, gam, b2, use_skip in ((0, 128, 0, False), (3, 100, -5, True), (-4, 131, 7, True), (200, -64, 1, False)):
        x0 = a / 128.0
        x1 = np.clip(x0 + b1 / 128.0, -127 / 128, 127 / 128)
        conv = ops.conv_fwd(d, np.rint(x1 * 128).astype(np.int8), w) / 16384.0
        x2 = np.rint(conv * 128) / 128                      # Q_a1 = Q
        x3 = (gam / 128.0) * x2
        x4 = x3 + b2 / 128.0 + (x0 if use_skip else 0.0)
        x5 = np.clip(np.rint(np.maximum(x4, 0) * 128) / 128, -127 / 128, 127 / 128)   # Q_a2 = CQ
        u = ops.pre_bias(a, b1)
        t = ops.q_a1(ops.conv_fwd(d, u, w))
        z = ops.post_conv(t, gam, b2, a if use_skip else None)
        y, mask = ops.relu_q_a2(z)
        assert np.array_equal(u, np.rint(x1 * 128))
        assert np.array_equal(t, np.rint(x2 * 128))
        assert np.array_equal(z, np.rint(x4 * 16384))
        assert np.array_equal(y, np.rint(x5 * 128))
        assert np.array_equal(mask, x4 > 0)


def test_epilogue_special_cases():
    t = np.arange(-300, 300, dtype=np.int64)
    y, mask = ops.relu_q_a2(ops.post_conv(t, 128, 0))
    assert np.array_equal(y, np.clip(np.maximum(t, 0), 0, 127))
    assert np.array_equal(mask, t > 0)
    # a value strictly between 0 and half a step is active but rounds to code 0
    z = np.array([1, 63, 64, 65, 192, -1, 0])
    y, mask = ops.relu_q_a2(z)
    assert y.tolist() == [0, 0, 0, 1, 2, 0, 0]
    assert mask.tolist() == [True, True, True, True, True, False, False]
    # wide shortcut (output of the 1x1 shortcut convolution) adds on the same grid as an int8 one
    t = np.array([5, -9, 1000])
    sk = np.array([7, 3, -2000])
    assert np.array_equal(ops.post_conv(t, 128, 0, sk), 128 * (t + sk))
    assert ops.pre_bias(np.array([120, -120, 5], dtype=np.int8), 10).tolist() == [127, -110, 15]
    assert ops.pre_bias(np.array([120, -120, 5], dtype=np.int8), -10).tolist() == [110, -127, -5]


def test_update_rules():
    W = np.array([-127, -3, 0, 5, 127], dtype=np.int8)
    # |update| < 2^-8 -> weights unchanged: g max 127 * 2^-12, lr 2^-4 -> 127*2^-16 < 2^-8
    g = np.array([127, -127, 64, -64, 1], dtype=np.int8)
    assert np.array_equal(ops.update_weights(W, g, -12, 1, 4), W)
    # update exactly j * 2^-7: g codes on grid 2^-7 after lr=1: u = SQ(g) = g (max code >= 91) -> delta = g
    g = np.array([100, -100, 3, -3, 120], dtype=np.int8)
    assert ops.update_delta(g, -7, 1, 0).tolist() == g.tolist()
    assert ops.update_weights(W, g, -7, 1, 0).tolist() == [-127, 97, -3, 8, 7]
    # exponent above the weight grid: left shift, then clamp
    assert ops.update_delta(g, -6, 1, 0).tolist() == (2 * g.astype(int)).tolist()
    assert ops.update_weights(W, g, -6, 1, 0).tolist() == [-127, 127, -6, 11, -113]
    # exponent below: round half to even; sign(delta W) = -sign(g)
    assert ops.update_delta(np.array([127, 126, 3, 2, 1, -1, -2, -3]), -8, 1, 0).tolist() == [64, 63, 2, 1, 0, 0, -1, -2]
    rng = np.random.default_rng(0)
    for _ in range(20):
        g = rng.integers(-127, 128, size=200).astype(np.int8)
        W = rng.integers(-127, 128, size=200).astype(np.int8)
        Eg, m, j = int(rng.integers(-16, -4)), int(rng.integers(1, 50)), int(rng.integers(-3, 6))
        W2 = ops.update_weights(W, g, Eg, m, j)
        assert W2.min() >= -127 and W2.max() <= 127
        dW = W2.astype(int) - W
        assert np.all(dW * np.sign(g) <= 0)
        # literal: u = SQ(lr*g) in real numbers, W - u rounded to the weight grid, clamped
        lr = m * 2.0 ** -j
        uc, Eu = oq.sq_real(lr * g.astype(np.float64) * 2.0 ** Eg)
        want = np.clip(W - np.rint(uc * 2.0 ** (Eu + 7)), -127, 127)
        assert np.array_equal(W2, want)
    # scalars: unclamped
    assert ops.update_scalar(128, 100, -7, 1, 0) == 28
    assert ops.update_scalar(-200, -127, -7, 1, 0) == -73


def test_scalar_gradient_is_sq_of_sum():
    assert ops.scalar_gradient([(300, -20)]) == (127, -19)      # 300 -> r=8 -> 150 -> clamp
    assert ops.scalar_gradient([(-100, -20)]) == (-100, -20)    # r=7: shift 0
    assert ops.scalar_gradient([(0, -20)]) == (0, -20)
    # two terms on different grids: 3*2^-10 + 5*2^-12 = 17 * 2^-12 -> r = 4 -> 17<<3 = 136 -> 127
    assert ops.scalar_gradient([(3, -10), (5, -12)]) == (127, -15)
    assert ops.scalar_gradient([(1, -10), (1, -12)]) == (127, -17)  # 5*2^-12: r=2 -> 5<<5 = 160 -> 127
    assert ops.scalar_gradient([(1, -10), (2, -12)]) == (96, -16)   # 6*2^-12: r=3 -> 6<<4 = 96


def test_fixup_init_rules():
    assert fixup.alpha(8, 2) == pytest.approx(8 ** -0.5)
    assert fixup.alpha(16, 3) == 0.5
    assert fixup.alpha(9, 2) == pytest.approx(1 / 3)
    assert fixup.alpha(1, 2) == 1.0 and fixup.alpha(1, 3) == 1.0
    assert fixup.alpha(54, 2) == pytest.approx(54 ** -0.5)
    assert fixup.init_gamma_code() == 128 and fixup.init_bias_code() == 0
    z = si.standard_normal(0, "probe.w", (64, 3, 3, 16))
    assert abs(z.mean()) < 0.02 and abs(z.std() - 1) < 0.02
    n = 16 * 9
    w = fixup.init_conv_real(z, n, fixup.alpha(9, 2))
    assert w.dtype == np.float32
    assert w.std() == pytest.approx(math.sqrt(2 / n) / 3, rel=0.03)
    c = fixup.init_conv_codes(z, n, fixup.alpha(9, 2))
    assert c.dtype == np.int8 and np.array_equal(c, np.clip(np.rint(w.astype(np.float64) * 128), -127, 127))
    assert (c.astype(float) / 128).std() == pytest.approx(math.sqrt(2 / n) / 3, rel=0.1)


def test_maxpool_brute_force_and_routing():
    a = si.uniform_int8(0, "pool.a", (2, 7, 9, 3), -5, 5)        # many ties
    y, arg = ops.maxpool_fwd(a)
    N, H, W, C = a.shape
    P, Q = y.shape[1:3]
    assert (P, Q) == (4, 5)
    e = si.uniform_int8(0, "pool.e", y.shape)
    want_d = np.zeros(a.shape, dtype=np.int64)
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                for c in range(C):
                    cells = [(r, s) for r in range(3) for s in range(3)
                             if 0 <= 2 * p + r - 1 < H and 0 <= 2 * q + s - 1 < W]
                    vals = [int(a[n, 2 * p + r - 1, 2 * q + s - 1, c]) for r, s in cells]
                    m = max(vals)
                    r, s = cells[vals.index(m)]              # first winner in scan order
                    assert y[n, p, q, c] == m and arg[n, p, q, c] == 3 * r + s
                    want_d[n, 2 * p + r - 1, 2 * q + s - 1, c] += int(e[n, p, q, c])
    d = ops.maxpool_bwd(e, arg, a.shape)
    assert np.array_equal(d, want_d)
    assert int(d.sum()) == int(e.astype(np.int64).sum())


def test_head_against_float_reference():
    rng = np.random.default_rng(3)
    N, F, J, HW = 5, 24, 7, 16
    gap = rng.integers(0, 127 * HW, size=(N, F)).astype(np.int32)
    Wfc = rng.normal(size=(J, F)) * 0.3
    bfc = rng.normal(size=J) * 0.1
    lab = rng.integers(0, J, size=N).astype(np.int32)
    loss, d, dW, db, logits = ops.head(gap, Wfc, bfc, lab, HW)
    feat = gap / (128.0 * HW)
    lg = feat @ Wfc.T + bfc
    assert np.allclose(logits, lg, rtol=1e-13, atol=1e-13)
    lse = np.log(np.exp(lg - lg.max(1, keepdims=True)).sum(1)) + lg.max(1)
    assert loss == pytest.approx(float(np.mean(lse - lg[np.arange(N), lab])), rel=1e-12)
    p = np.exp(lg - lse[:, None])
    dl = (p - np.eye(J)[lab]) / N
    assert np.allclose(d, (dl @ Wfc) / HW, rtol=1e-6, atol=1e-12)        # fp32 output
    assert np.allclose(dW, dl.T @ feat, rtol=1e-11, atol=1e-14)
    assert np.allclose(db, dl.sum(0), rtol=1e-11, atol=1e-14)
    lib = ops.lib()
    for x in [0.0, -1e-9, -0.3, -1.0, -17.25, -300.0, -699.0]:
        assert lib.eo_head_exp(x) == pytest.approx(math.exp(x), rel=4e-16)


def test_stochastic_rounding_of_the_update():
    """The optional stochastic rounding (beyond the paper, off by default): hand cases with given hash words, the
    two-neighbour bracket, exactness for left shifts, zero bias, and the generator against a scalar re-evaluation of its
    definition."""
    from oracle import ops as oo
    # d = floor((v + r) / 2^s), r = word mod 2^s
    assert oo.sr_shift(np.array([5, 5, -5, -5, 16, 0]), 3, np.array([2, 3, 2, 5, 7, 7])).tolist() == [0, 1, -1, 0, 2, 0]
    assert oo.sr_shift(np.array([3, -3]), 0, np.array([99, 99])).tolist() == [3, -3]
    assert oo.sr_shift(np.array([3, -3]), -4, np.array([99, 99])).tolist() == [48, -48]
    # only the low s bits of the word count; a shift beyond 62 is capped
    assert oo.sr_shift(np.array([5]), 3, np.array([2 + 8 * 12345], dtype=np.uint64)).tolist() == [0]
    assert oo.sr_shift(np.array([127, -127]), 70, np.array([2 ** 62 - 1, 0], dtype=np.uint64)).tolist() == [1, -1]
    # generator: one element re-evaluated with Python integers
    seed, tensor, step, idx = 7, 0xDEADBEEF, 41, 1234567
    M = (1 << 64) - 1
    z = (seed * oo.SR_A + tensor * oo.SR_B + step * oo.SR_C + idx * oo.SR_D) & M
    z ^= z >> 30; z = (z * 0xBF58476D1CE4E5B9) & M
    z ^= z >> 27; z = (z * 0x94D049BB133111EB) & M
    z ^= z >> 31
    w = oo.sr_words(seed, tensor, step, idx + 1)
    assert int(w[idx]) == z and len(set(w[:1000].tolist())) == 1000
    # bracket and zero bias: v / 2^s lies between the two candidates, the mean over many draws approaches it
    v = np.full(200000, 37, dtype=np.int64)
    d = oo.sr_shift(v, 6, oo.sr_words(1, 2, 3, v.size))
    assert set(d.tolist()) == {0, 1} and abs(d.mean() - 37 / 64) < 0.005
    d = oo.sr_shift(-v, 6, oo.sr_words(1, 2, 4, v.size))
    assert set(d.tolist()) == {-1, 0} and abs(d.mean() + 37 / 64) < 0.005
    # whole update: deterministic rounding loses a sub-code update, the stochastic one keeps its mean
    W = np.zeros(100000, dtype=np.int8)
    g = np.full(100000, 100, dtype=np.int8)                 # the gradient 100 * 2^-17 is a tenth of a code
    assert not oo.update_weights(W, g, -17, 1, 0).any()
    Ws = oo.update_weights(W, g, -17, 1, 0, sr=(5, 6, 7))
    from oracle.quant import sq_int
    uc, Eu = sq_int(np.array([100]), -17)                  # Q_u: (100, -17) -> the update in codes is uc * 2^(Eu+7)
    assert set(Ws.tolist()) == {-1, 0}
    assert abs(-Ws.astype(np.float64).mean() - float(uc[0]) * 2.0 ** (Eu + 7)) < 0.01
