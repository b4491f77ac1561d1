"""Pin of the oracle's backward pass and update on a tiny two-block network: Eq.3 (error chain), Eq.4 (parameter
gradients), Eq.11-13 (Q_e, Q_g, Q_u) and Eq.8 / Eq.10 (Q_w, Q_b, Q_gamma) evaluated LITERALLY in exact rational
arithmetic -- real values, the scale quantiser with its printed log2 / division / clamp, transposed convolutions as
plain loops over the definition -- and compared with the oracle's integer formulation code by code and exponent by
exponent.  A dropped term, a wrong exponent offset, a shift aligned the wrong way, the wrong error fed to the
shortcut or a scalar sum taken on the wrong grid changes at least one of them.

The forward quantities the backward pass consumes (x1, x2, the ReLU masks) and the error leaving the float head are
taken from the oracle's trace: they are pinned elsewhere (exact agreement with a straight-through autograd model).
What stays a reading of the paper, and cannot be pinned, is the block-level wiring itself (which the literal
evaluation below spells out once more): the shortcut receives the error after the last ReLU of the block, and the
two errors meeting at a block input are each quantised first and then quantised again after their exact sum.
"""
import math
from fractions import Fraction

import numpy as np

import seeded_inputs as si
from oracle.net import Net

F = Fraction
CFG = dict(block="basic", depths=(1, 1), widths=(4, 8), stem="cifar", classes=5, in_hw=8, in_ch=3)


# ---- the printed quantisers (Section 3.2.2), k = 8 ----
def R(fr: Fraction) -> int:
    fl = math.floor(fr)
    d = fr - fl
    return fl + 1 if (d > F(1, 2) or (d == F(1, 2) and fl % 2 == 1)) else fl


def Q(x):
    return F(R(x * 128), 128)


def CQ(x):
    return max(F(-127, 128), min(F(127, 128), Q(x)))


def SQ(xs):
    """xs: object array of Fractions -> (quantised values, scale); all-zero input passes through."""
    flat = [abs(v) for v in xs.reshape(-1)]
    m = max(flat)
    if m == 0:
        return xs.copy(), None
    lg = math.log2(float(m))
    assert abs((lg % 1.0) - 0.5) > 1e-9                     # no tie in R(log2 .) for these inputs
    scale = F(2) ** round(lg)
    out = np.empty(xs.shape, dtype=object)
    of = out.reshape(-1)
    for i, v in enumerate(xs.reshape(-1)):
        of[i] = scale * CQ(v / scale)
    return out, scale


def frac_array(codes, E):
    out = np.empty(codes.shape, dtype=object)
    of = out.reshape(-1)
    s = F(2) ** int(E)
    for i, c in enumerate(np.asarray(codes).reshape(-1)):
        of[i] = int(c) * s
    return out


def same(values, scale, codes, E, what):
    """Literal SQ output (values, scale) against the oracle's (int8 codes, exponent)."""
    if scale is None:                                       # all zero: the oracle keeps the incoming exponent
        assert not np.asarray(codes).any(), what
        return
    assert scale == F(2) ** (int(E) + 7), (what, scale, E)
    got = [v / scale * 128 for v in values.reshape(-1)]
    assert got == [int(c) for c in np.asarray(codes).reshape(-1)], what


# ---- transposed convolutions by their definition ----
def conv_T_data(d, e3, W):
    out = np.full((d.N, d.H, d.W, d.C), F(0), dtype=object)
    for n in range(d.N):
        for p in range(d.P):
            for q in range(d.Q):
                for r in range(d.R):
                    for s in range(d.S):
                        h, x = p * d.stride + r - d.pad, q * d.stride + s - d.pad
                        if 0 <= h < d.H and 0 <= x < d.W:
                            for k in range(d.K):
                                if e3[n, p, q, k] != 0:
                                    out[n, h, x, :] = out[n, h, x, :] + e3[n, p, q, k] * W[k, r, s, :]
    return out


def conv_T_weight(d, e3, x1):
    out = np.full((d.K, d.R, d.S, d.C), F(0), dtype=object)
    for n in range(d.N):
        for p in range(d.P):
            for q in range(d.Q):
                for r in range(d.R):
                    for s in range(d.S):
                        h, x = p * d.stride + r - d.pad, q * d.stride + s - d.pad
                        if 0 <= h < d.H and 0 <= x < d.W:
                            for k in range(d.K):
                                if e3[n, p, q, k] != 0:
                                    out[k, r, s, :] = out[k, r, s, :] + e3[n, p, q, k] * x1[n, h, x, :]
    return out


def total(a):
    return sum(a.reshape(-1), F(0))


def test_backward_and_update_equal_the_literal_formulas():
    N = 2
    net = Net(CFG, N, seed=3)
    # multipliers and biases off their initial values, so that every term of Eq.3 / Eq.4 matters
    for i, k in enumerate(sorted(net.scal)):
        net.scal[k] += (i % 7) - 3
    net.scal["s0b0.g"], net.scal["s1b0.g"] = 117, -77
    x = si.batch_images(3, 0, N, CFG["in_hw"])
    lab = si.batch_labels(3, 0, N, CFG["classes"])
    W_before = {k: v.copy() for k, v in net.W.items()}
    s_before = dict(net.scal)
    lr_m, lr_j = 3, -3                                      # lr = 24: weight codes do move
    lr = F(lr_m) * F(2) ** (-lr_j)
    net.step(x, lab, lr_m, lr_j)
    T = net.trace
    Wr = {k: frac_array(v, -7) for k, v in W_before.items()}

    scal_sums = {}          # parameter -> list of real sums (Eq.4 before Q_g)
    gw = {}                 # layer -> literal Q_g output (values, scale)

    def layer_backward(u, e0, need_dx=True):
        """Eq.3 / Eq.4 for one layer; e0 real-valued.  Returns (e4, e1)."""
        c = u.cache
        e1 = e0 * c["mask"].astype(int) if u.relu else e0                    # e1 = e0 * relu'(x4)
        if u.relu:
            scal_sums.setdefault(u.b_post, []).append(total(e1))            # g_b2 = Q_g(e1), summed
        e2 = e1
        if u.gamma:
            x2 = frac_array(c["t"], -7)
            scal_sums.setdefault(u.gamma, []).append(total(e2 * x2))        # g_gamma = Q_g(e2 * x2), summed
            e3, sc3 = SQ(e2 * F(s_before[u.gamma], 128))                    # e3 = Q_e(e2 * gamma)
            same(e3, sc3, T[u.name + ".e3"], T[u.name + ".E3"], u.name + ".e3")
        else:
            e3 = e2
        x1 = frac_array(c["x1"], -7)
        gw[u.name] = SQ(conv_T_weight(u.shape, e3, x1))                     # g_w = Q_g(e3 * x1)
        same(*gw[u.name], T[u.name + ".gw"], T[u.name + ".Eg"], u.name + ".gw")
        if not need_dx:
            return None, e1
        e4, sc4 = SQ(conv_T_data(u.shape, e3, Wr[u.name]))                  # e4 = Q_e(e3 * W)
        same(e4, sc4, T[u.name + ".e4"], T[u.name + ".E4"], u.name + ".e4")
        return e4, e1

    e = frac_array(T["head.e"], T["head.E"])
    for b in reversed(net.blocks):
        e_skip = None
        for i in range(len(b.units) - 1, -1, -1):
            u = b.units[i]
            e4, e1 = layer_backward(u, e)
            if i == len(b.units) - 1:
                e_skip = e1                                                  # the shortcut leaves after the last ReLU
            scal_sums.setdefault(u.b_pre, []).append(total(e4))             # g_b1 = Q_g(e4), summed
            e = e4
        if b.ds is not None:
            e4d, _ = layer_backward(b.ds, e_skip)
            scal_sums[b.units[0].b_pre].append(total(e4d))                  # the shortcut convolution shares x1
            e, sc = SQ(e + e4d)
        else:
            e, sc = SQ(e + e_skip)
        same(e, sc, T[b.name + ".e_in"], T[b.name + ".E_in"], b.name + ".e_in")
    layer_backward(net.stem, e, need_dx=False)

    # ---- scalar gradients: Q_g of the one-element tensor; then Q_u and the unclamped update (Eq.10, Eq.13)
    assert set(scal_sums) == set(s_before)
    for name, terms in scal_sums.items():
        g, sc = SQ(np.array([sum(terms, F(0))], dtype=object))
        same(g, sc, np.array([T[name + ".gs"]]), T[name + ".Egs"], name + ".gs")
        upd, _ = SQ(lr * g)
        new = Q(F(s_before[name], 128) - upd[0])
        assert new * 128 == net.scal[name], name
    # ---- weights: W <- Q_w(W - Q_u(lr * g_w))  (Eq.13, Eq.8)
    moved = 0
    for name, (g, sc) in gw.items():
        upd, _ = SQ(lr * g)
        want = [CQ(w - d) * 128 for w, d in zip(Wr[name].reshape(-1), upd.reshape(-1))]
        assert want == [int(c) for c in net.W[name].reshape(-1)], name
        moved += int((net.W[name] != W_before[name]).sum())
    assert moved > 50, "no weight code moved: the update comparison would be vacuous"
