"""Pins for the oracle's whole-network step: topology counts that are textbook values,
an independent PyTorch-autograd model with straight-through quantisers (forward must
agree exactly, gradients closely), and exponent equivariance of the backward chain."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import seeded_inputs as si
from oracle.net import Net


def macs(net):
    tot = 0
    units = [net.stem] + [u for b in net.blocks for u in b.units] + [b.ds for b in net.blocks if b.ds]
    for u in units:
        d = u.shape
        tot += d.P * d.Q * d.K * d.C * d.R * d.S
    return tot, len(units)


def test_topology_counts():
    # conv counts and per-image multiply-accumulates of the standard architectures
    n, c = macs(Net(si.WORKLOADS["resnet20"], 1))
    assert c == 21 and n == pytest.approx(40.8e6, rel=0.01)
    n, c = macs(Net(si.WORKLOADS["resnet18"], 1))
    assert c == 20 and n == pytest.approx(1.814e9, rel=0.005)
    n, c = macs(Net(si.WORKLOADS["resnet50"], 1))
    assert c == 53 and n == pytest.approx(4.087e9, rel=0.005)
    net = Net(si.WORKLOADS["resnet50"], 1)
    assert net.L == 16 and net.m == 3 and net.out_hw == 7 and net.out_ch == 2048
    assert sum(v.size for v in net.W.values()) == pytest.approx(23.5e6, rel=0.01)
    assert len(net.scal) == 16 * 7 + 1
    net = Net(si.WORKLOADS["resnet20"], 1)
    assert net.L == 9 and net.out_hw == 8 and len(net.scal) == 9 * 5 + 1


# ---------------- independent straight-through model in PyTorch (fp64, exact on dyadics) ----------------
class _Round(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x):
        return torch.round(x)          # half to even

    @staticmethod
    def backward(ctx, g):
        return g


def tQ(x):
    return _Round.apply(x * 128) / 128


def tCQ(x):
    q = tQ(x)
    return q + (torch.clamp(q, -127 / 128, 127 / 128) - q).detach()


def t_unit(net, P, u, x0, skip=None):
    x1 = x0
    if u.b_pre:
        x1 = x0 + P[u.b_pre]
        x1 = x1 + (torch.clamp(x1, -127 / 128, 127 / 128) - x1).detach()
    x2 = tQ(F.conv2d(x1, P[u.name], stride=u.shape.stride, padding=u.shape.pad))
    if not u.relu:
        return x2
    x3 = P[u.gamma] * x2 if u.gamma else x2
    x4 = x3 + P[u.b_post] + (skip if skip is not None else 0)
    return tCQ(torch.relu(x4))


def torch_model(net, x_f32, labels):
    P = {}
    for k, w in net.W.items():
        P[k] = torch.tensor(w.astype(np.float64) / 128).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    for k, v in net.scal.items():
        P[k] = torch.tensor(v / 128.0, dtype=torch.float64, requires_grad=True)
    Wfc = torch.tensor(net.Wfc, requires_grad=True)
    bfc = torch.tensor(net.bfc, requires_grad=True)
    x = torch.tensor(x_f32.astype(np.float64)).permute(0, 3, 1, 2)
    a = tCQ(x * 0.25)
    acts = {}
    y = t_unit(net, P, net.stem, a)
    if net.pool:
        y = F.max_pool2d(y, 3, 2, 1)
    for b in net.blocks:
        h, skip = y, y
        for i, u in enumerate(b.units):
            last = i == len(b.units) - 1
            if i == 0 and b.ds is not None:
                x1 = y + P[u.b_pre]
                x1 = x1 + (torch.clamp(x1, -127 / 128, 127 / 128) - x1).detach()
                skip = t_unit(net, P, b.ds, x1)
            h = t_unit(net, P, u, h, skip if last else None)
            acts[u.name] = h
        y = h
    feat = y.mean(dim=(2, 3))
    logits = feat @ Wfc.T + bfc
    loss = F.cross_entropy(logits, torch.tensor(labels, dtype=torch.long))
    loss.backward()
    return loss.item(), logits.detach().numpy(), acts, P, Wfc, bfc


@pytest.mark.parametrize("wl,N", [("tiny_basic", 4), ("tiny_bottleneck", 3)])
def test_against_straight_through_autograd(wl, N):
    cfg = si.WORKLOADS[wl]
    net = Net(cfg, N, seed=1)
    # move the scalars off their initial values so that every term is exercised
    for i, k in enumerate(sorted(net.scal)):
        net.scal[k] += (i % 5) - 2
    x = si.batch_images(1, 0, N, cfg["in_hw"])
    lab = si.batch_labels(1, 0, N, cfg["classes"])
    tl, tlogits, tacts, P, tWfc, tbfc = torch_model(net, x, lab)
    W0 = {k: v.copy() for k, v in net.W.items()}
    s0 = dict(net.scal)
    Wfc0 = net.Wfc.copy()
    loss = net.step(x, lab, 1, 0)
    T = net.trace
    # forward: exact
    for name, act in tacts.items():
        want = np.rint(act.detach().permute(0, 2, 3, 1).numpy() * 128)
        assert np.array_equal(T[name + ".y"], want), name
    assert np.allclose(T["head.logits"], tlogits, rtol=1e-12, atol=1e-12)
    assert loss == pytest.approx(tl, rel=1e-10)
    # float head gradient (lr = 1): W' = W - dW
    assert np.allclose(Wfc0 - net.Wfc, tWfc.grad.numpy(), rtol=1e-9, atol=1e-13)
    # backward: quantised errors vs exact straight-through gradients
    worst = 1.0
    for k in W0:
        g = T[k + ".gw"].astype(np.float64) * 2.0 ** T[k + ".Eg"]
        tg = P[k].grad.permute(0, 2, 3, 1).numpy()
        cos = float((g * tg).sum() / (np.linalg.norm(g) * np.linalg.norm(tg) + 1e-300))
        ratio = np.linalg.norm(g) / (np.linalg.norm(tg) + 1e-300)
        worst = min(worst, cos)
        assert cos > 0.9, (k, cos)
        assert 0.6 < ratio < 1.5, (k, ratio)
    # scalar gradients: sign and magnitude (one-element SQ keeps them within sqrt2 of a power of two)
    for k in s0:
        g = T[k + ".gs"] * 2.0 ** T[k + ".Egs"]
        tg = float(P[k].grad)
        if abs(tg) > 1e-4:
            assert np.sign(g) == np.sign(tg), k
            assert 0.4 < g / tg < 2.5, (k, g, tg)


def test_backward_chain_is_exponent_equivariant():
    # for a fixed forward pass the backward chain is linear in the incoming error: raising its exponent
    # by one must leave every int8 code alone and raise every downstream exponent by one
    cfg = si.WORKLOADS["block16"]
    outs = []
    for E0 in (-7, -6, -11):
        net = Net(cfg, 2, seed=0)
        net.scal["s0b0.g"] = 117
        net.scal["s0b0.b2a"] = -3
        a = si.uniform_int8(0, "a", (2, 32, 32, 16))
        e0 = si.uniform_int8(0, "e0", (2, 32, 32, 16))
        net.block_step(a, e0, E0, 1, 40)       # tiny lr: parameters do not move
        outs.append(dict(net.trace))
    base = outs[0]
    for o, dE in ((outs[1], 1), (outs[2], -4)):
        for k, v in base.items():
            if isinstance(v, np.ndarray):
                assert np.array_equal(v, o[k]), k
            elif k.endswith((".E3", ".E4", ".Eg", ".E_in", ".Egs")):
                assert o[k] == v + dE, k
            else:
                assert o[k] == v, k
