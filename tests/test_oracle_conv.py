"""Pins for the oracle's three convolutions (Eq.2 conv, Eq.3 e4, Eq.4 g_w): brute force
on tiny tensors, the adjoint identity in exact integers, library special cases,
and the int32 overflow bound."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import ops
from oracle.ops import ConvShape

SHAPES = [
    ConvShape(2, 5, 6, 3, 4, 3, 3, 1, 1),
    ConvShape(1, 7, 7, 5, 3, 3, 3, 2, 1),
    ConvShape(2, 6, 5, 4, 6, 1, 1, 1, 0),
    ConvShape(2, 6, 6, 4, 5, 1, 1, 2, 0),
    ConvShape(1, 11, 12, 3, 2, 7, 7, 2, 3),
    ConvShape(1, 4, 4, 2, 2, 3, 3, 1, 0),
    ConvShape(1, 8, 8, 2, 3, 3, 3, 2, 0),
]


def rand_i8(name, shape, seed=0):
    return si.uniform_int8(seed, name, shape)


def brute_conv(d, u, w):
    acc = np.zeros((d.N, d.P, d.Q, d.K), dtype=np.int64)
    for n in range(d.N):
        for p in range(d.P):
            for q in range(d.Q):
                for k in range(d.K):
                    for r in range(d.R):
                        for s in range(d.S):
                            for c in range(d.C):
                                h, x = p * d.stride + r - d.pad, q * d.stride + s - d.pad
                                if 0 <= h < d.H and 0 <= x < d.W:
                                    acc[n, p, q, k] += int(u[n, h, x, c]) * int(w[k, r, s, c])
    return acc


@pytest.mark.parametrize("d", SHAPES)
def test_fwd_brute_force_and_torch(d):
    u, w = rand_i8("u", (d.N, d.H, d.W, d.C)), rand_i8("w", (d.K, d.R, d.S, d.C))
    acc = ops.conv_fwd(d, u, w)
    assert np.array_equal(acc, brute_conv(d, u, w))
    # library routine: torch conv2d in fp64 is exact on these integers
    t = torch.nn.functional.conv2d(torch.from_numpy(u.astype(np.float64)).permute(0, 3, 1, 2),
                                   torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2),
                                   stride=d.stride, padding=d.pad)
    assert np.array_equal(acc, t.permute(0, 2, 3, 1).numpy().astype(np.int64))


@pytest.mark.parametrize("d", SHAPES)
def test_adjoint_identity(d):
    # <conv(u,W), e> = <u, dX(e,W)> = <W, dW(e,u)> exactly: pins both backward convolutions
    u, w = rand_i8("u", (d.N, d.H, d.W, d.C)), rand_i8("w", (d.K, d.R, d.S, d.C))
    e = rand_i8("e", (d.N, d.P, d.Q, d.K))
    lhs = int((ops.conv_fwd(d, u, w).astype(np.int64) * e).sum())
    dx = ops.conv_bwd_data(d, e, w)
    g = ops.conv_bwd_weight(d, e, u)
    assert int((dx.astype(np.int64) * u).sum()) == lhs
    assert int((g.astype(np.int64) * w).sum()) == lhs


@pytest.mark.parametrize("d", SHAPES)
def test_backward_against_basis_probes(d):
    # every entry of dX / dW is the coefficient of one input / weight in <conv, e>: probe a few with unit tensors
    rng = np.random.default_rng(7)
    u, w = rand_i8("u", (d.N, d.H, d.W, d.C)), rand_i8("w", (d.K, d.R, d.S, d.C))
    e = rand_i8("e", (d.N, d.P, d.Q, d.K))
    dx = ops.conv_bwd_data(d, e, w)
    g = ops.conv_bwd_weight(d, e, u)
    for _ in range(6):
        idx = tuple(int(rng.integers(0, s)) for s in u.shape)
        unit = np.zeros_like(u)
        unit[idx] = 1
        assert int((ops.conv_fwd(d, unit, w).astype(np.int64) * e).sum()) == int(dx[idx])
        idx = tuple(int(rng.integers(0, s)) for s in w.shape)
        unit = np.zeros_like(w)
        unit[idx] = 1
        assert int((ops.conv_fwd(d, u, unit).astype(np.int64) * e).sum()) == int(g[idx])


def test_1x1_is_integer_gemm():
    d = ConvShape(3, 5, 4, 24, 10, 1, 1, 1, 0)
    u, w = rand_i8("u", (d.N, d.H, d.W, d.C)), rand_i8("w", (d.K, 1, 1, d.C))
    want = u.reshape(-1, d.C).astype(np.int64) @ w.reshape(d.K, d.C).astype(np.int64).T
    assert np.array_equal(ops.conv_fwd(d, u, w).reshape(-1, d.K), want)
    e = rand_i8("e", (d.N, d.P, d.Q, d.K))
    assert np.array_equal(ops.conv_bwd_data(d, e, w).reshape(-1, d.C),
                          e.reshape(-1, d.K).astype(np.int64) @ w.reshape(d.K, d.C).astype(np.int64))
    assert np.array_equal(ops.conv_bwd_weight(d, e, u).reshape(d.K, d.C),
                          e.reshape(-1, d.K).astype(np.int64).T @ u.reshape(-1, d.C).astype(np.int64))


def test_centre_delta_kernel_is_identity():
    d = ConvShape(2, 6, 6, 4, 4, 3, 3, 1, 1)
    u = rand_i8("u", (d.N, d.H, d.W, d.C))
    w = np.zeros((4, 3, 3, 4), dtype=np.int8)
    for k in range(4):
        w[k, 1, 1, k] = 1
    assert np.array_equal(ops.conv_fwd(d, u, w), u.astype(np.int32))


def test_int32_bound_is_detected():
    # reduction length N*P*Q: fits int32 iff <= floor((2^31-1)/127^2) = 133144 in the worst case
    assert (2 ** 31 - 1) // (127 * 127) == 133144
    n_ok, n_bad = 133144, 133145
    for n, expect_bad in ((n_ok, 0), (n_bad, 1)):
        d = ConvShape(1, 1, n, 1, 1, 1, 1, 1, 0)
        u = np.full((1, 1, n, 1), 127, dtype=np.int8)
        e = np.full((1, 1, n, 1), 127, dtype=np.int8)
        g = np.empty((1, 1, 1, 1), dtype=np.int32)
        import ctypes as C
        bad = ops.lib().eo_conv_bwd_weight(C.byref(d.c()), ops._p(e), ops._p(u), ops._p(g))
        assert bad == expect_bad
    # forward / backward-data reductions of the nets used here are far below the bound
    assert 127 * 127 * 4608 < 2 ** 31 - 1
