"""Oracle: a whole Fixup residual network trained for one full-int8 step.
TEST INFRASTRUCTURE ONLY -- see the package docstring.

Layer arithmetic follows Eq.2-4 and Eq.8-13; the block topology (where the
shortcut is added, one multiplier per block, a bias in front of every
convolution and every ReLU, 1x1 strided convolution on the biased input when
the shape changes) is that of the Fixup residual block the paper builds on
(Section 3.1).  Every intermediate tensor is kept in `trace` under a stable
name so that tests can compare them one by one.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field

import numpy as np

import seeded_inputs as si

from . import fixup, ops
from .ops import ConvShape
from .quant import cq_code, sq_real


@dataclass
class Unit:
    """One Fixup layer of Eq.2: (pre-bias) conv, Q_a1, (multiplier), post-bias, (+shortcut), ReLU, Q_a2."""
    name: str
    shape: ConvShape
    b_pre: str | None
    gamma: str | None
    b_post: str | None
    relu: bool = True
    cache: dict = field(default_factory=dict)


@dataclass
class Block:
    name: str
    units: list          # main branch, in forward order
    ds: Unit | None      # 1x1 strided shortcut convolution (no bias of its own, output kept wide)


class Net:
    def __init__(self, cfg: dict, batch: int, seed: int = 0, sr_seed: int | None = None):
        self.cfg, self.N, self.seed = dict(cfg), batch, seed
        self.sr_seed, self.sr_step = sr_seed, 0      # optional stochastic rounding of the update (beyond the paper)
        self.W: dict[str, np.ndarray] = {}       # int8 KRSC codes
        self.scal: dict[str, int] = {}           # bias / multiplier codes (grid 2^-7)
        self.trace: dict[str, object] = {}
        bt = cfg["block"]
        self.m = 2 if bt == "basic" else 3
        self.L = int(sum(cfg["depths"]))
        a = fixup.alpha(self.L, self.m)
        hw, ch = cfg["in_hw"], cfg["in_ch"]
        # ---- stem
        self.stem = None
        self.pool = False
        if cfg["stem"] == "cifar":
            w0 = cfg["widths"][0]
            self.stem = Unit("stem", ConvShape(batch, hw, hw, ch, w0, 3, 3, 1, 1), None, None, "stem.b")
            ch = w0
        elif cfg["stem"] == "imagenet":
            w0 = cfg["widths"][0]
            self.stem = Unit("stem", ConvShape(batch, hw, hw, ch, w0, 7, 7, 2, 3), None, None, "stem.b")
            hw = self.stem.shape.P
            self.pool = True
            hw = (hw + 2 - 3) // 2 + 1
            ch = w0
        if self.stem is not None:
            self._init_conv(self.stem, 1.0)
            self.scal["stem.b"] = fixup.init_bias_code()
        # ---- residual stages
        self.blocks: list[Block] = []
        for si_, (depth, width) in enumerate(zip(cfg["depths"], cfg["widths"])):
            for bi in range(depth):
                stride = 2 if (bi == 0 and si_ > 0) else 1
                out_ch = width if bt == "basic" else 4 * width
                nm = f"s{si_}b{bi}"
                units = []
                if bt == "basic":
                    units.append(Unit(nm + ".c1", ConvShape(batch, hw, hw, ch, width, 3, 3, stride, 1),
                                      nm + ".b1a", None, nm + ".b1b"))
                    h2 = units[0].shape.P
                    units.append(Unit(nm + ".c2", ConvShape(batch, h2, h2, width, width, 3, 3, 1, 1),
                                      nm + ".b2a", nm + ".g", nm + ".b2b"))
                else:
                    units.append(Unit(nm + ".c1", ConvShape(batch, hw, hw, ch, width, 1, 1, 1, 0),
                                      nm + ".b1a", None, nm + ".b1b"))
                    units.append(Unit(nm + ".c2", ConvShape(batch, hw, hw, width, width, 3, 3, stride, 1),
                                      nm + ".b2a", None, nm + ".b2b"))
                    h2 = units[1].shape.P
                    units.append(Unit(nm + ".c3", ConvShape(batch, h2, h2, width, out_ch, 1, 1, 1, 0),
                                      nm + ".b3a", nm + ".g", nm + ".b3b"))
                ds = None
                if stride != 1 or ch != out_ch:
                    ds = Unit(nm + ".ds", ConvShape(batch, hw, hw, ch, out_ch, 1, 1, stride, 0), None, None, None,
                              relu=False)
                    self._init_conv(ds, 1.0)
                for u in units:
                    self._init_conv(u, a)
                    for s in (u.b_pre, u.b_post):
                        self.scal[s] = fixup.init_bias_code()
                    if u.gamma:
                        self.scal[u.gamma] = fixup.init_gamma_code()
                self.blocks.append(Block(nm, units, ds))
                hw, ch = units[-1].shape.P, out_ch
        self.out_hw, self.out_ch = hw, ch
        # ---- float head
        self.classes = cfg["classes"]
        if self.classes:
            z = si.standard_normal(seed, "fc.w", (self.classes, ch))
            self.Wfc = z * fixup.kaiming_std(ch)
            self.bfc = np.zeros(self.classes, dtype=np.float64)

    def _init_conv(self, u: Unit, scale: float):
        d = u.shape
        z = si.standard_normal(self.seed, u.name + ".w", (d.K, d.R, d.S, d.C))
        self.W[u.name] = fixup.init_conv_codes(z, d.C * d.R * d.S, scale)

    # ------------------------------------------------------------------ forward
    def _unit_fwd(self, u: Unit, a, skip=None):
        """Eq.2 for one layer.  `a` is x0 (int8 codes)."""
        T = self.trace
        x1 = ops.pre_bias(a, self.scal[u.b_pre]) if u.b_pre else a
        acc = ops.conv_fwd(u.shape, x1, self.W[u.name])
        t = ops.q_a1(acc)
        u.cache = dict(x1=x1, t=t)
        T[u.name + ".u"] = x1
        if not u.relu:                       # shortcut convolution: wide Q_a1 output is the result
            T[u.name + ".t"] = t
            return t
        g = self.scal[u.gamma] if u.gamma else fixup.init_gamma_code()
        z = ops.post_conv(t, g, self.scal[u.b_post], skip)
        y, mask = ops.relu_q_a2(z)
        u.cache["mask"] = mask
        T[u.name + ".y"], T[u.name + ".mask"] = y, mask
        if u.gamma:
            T[u.name + ".t"] = t
        return y

    def forward_blocks(self, a):
        for b in self.blocks:
            h = a
            skip = a
            for i, u in enumerate(b.units):
                last = i == len(b.units) - 1
                if i == 0 and b.ds is not None:
                    # the shortcut convolution reads the same biased input as the first layer
                    x1 = ops.pre_bias(a, self.scal[u.b_pre])
                    skip = self._unit_fwd(b.ds, x1)
                h = self._unit_fwd(u, h, skip if last else None)
            a = h
        return a

    def forward(self, x_f32):
        """Network input -> CQ(x/4) (codes clamp(R(32x))), stem, blocks, integer pooled sums."""
        T = self.trace
        a = cq_code(np.asarray(x_f32, dtype=np.float64) * 0.25).astype(np.int8)
        T["in.a"] = a
        y = self._unit_fwd(self.stem, a)
        if self.pool:
            T["stem.prepool"] = y
            y, arg = ops.maxpool_fwd(y)
            self.stem.cache["arg"], self.stem.cache["prepool_shape"] = arg, T["stem.prepool"].shape
            T["pool.y"] = y
        y = self.forward_blocks(y)
        gap = y.astype(np.int64).sum(axis=(1, 2)).astype(np.int32)
        T["gap.sum"] = gap
        return y, gap

    # ------------------------------------------------------------------ backward
    def _unit_bwd(self, u: Unit, e0, E0, grads, sums, need_dx=True):
        """Eq.3 / Eq.4 for one layer.  Returns (e4, E4, e1) -- e1 is what the shortcut receives."""
        T = self.trace
        c = u.cache
        if u.relu:
            e1 = (e0.astype(np.int64) * c["mask"]).astype(np.int8)
            sums.setdefault(u.b_post, []).append((int(e1.astype(np.int64).sum()), E0))
        else:
            e1 = e0
        if u.gamma:
            sums.setdefault(u.gamma, []).append((int((e1.astype(np.int64) * c["t"]).sum()), E0 - 7))
            e3, E3 = ops.sq_error_gamma(e1, E0, self.scal[u.gamma])
        else:
            e3, E3 = e1, E0
        T[u.name + ".e3"], T[u.name + ".E3"] = e3, E3
        G = ops.conv_bwd_weight(u.shape, e3, c["x1"])
        grads[u.name] = ops.sq_acc(G, E3 - 7)
        T[u.name + ".G"] = G
        T[u.name + ".gw"], T[u.name + ".Eg"] = grads[u.name]
        if not need_dx:
            return None, None, e1
        D = ops.conv_bwd_data(u.shape, e3, self.W[u.name])
        e4, E4 = ops.sq_acc(D, E3 - 7)
        T[u.name + ".e4"], T[u.name + ".E4"] = e4, E4
        return e4, E4, e1

    def backward_blocks(self, e, E, grads, sums):
        T = self.trace
        for b in reversed(self.blocks):
            e_sk, E_sk = None, None
            for i in range(len(b.units) - 1, -1, -1):
                u = b.units[i]
                e4, E4, e1 = self._unit_bwd(u, e, E, grads, sums)
                if i == len(b.units) - 1:
                    e_sk, E_sk = e1, E
                sums.setdefault(u.b_pre, []).append((int(e4.astype(np.int64).sum()), E4))
                e, E = e4, E4
            first = b.units[0]
            if b.ds is not None:
                e4d, E4d, _ = self._unit_bwd(b.ds, e_sk, E_sk, grads, sums)
                sums[first.b_pre].append((int(e4d.astype(np.int64).sum()), E4d))
                e, E = ops.merge_errors(e, E, e4d, E4d)
            else:
                e, E = ops.merge_errors(e, E, e_sk, E_sk)
            T[b.name + ".e_in"], T[b.name + ".E_in"] = e, E
        return e, E

    def backward_stem(self, e, E, grads, sums):
        T = self.trace
        if self.pool:
            d = ops.maxpool_bwd(e, self.stem.cache["arg"], self.stem.cache["prepool_shape"])
            e, E = ops.sq_acc(d, E)
            T["pool.e"], T["pool.E"] = e, E
        self._unit_bwd(self.stem, e, E, grads, sums, need_dx=False)

    # ------------------------------------------------------------------ update
    def apply_updates(self, grads, sums, lr_m, lr_j):
        """Eq.13 on every parameter; all gradients were taken with the old parameters.  With self.sr_seed set (not
        the paper's method: see ops.sr_shift) the update is rounded stochastically; a tensor's id in the hash is the
        CRC-32 of its name, the step counter advances once per call."""
        T = self.trace
        sr = (lambda name: None) if self.sr_seed is None else \
             (lambda name: (self.sr_seed, zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF, self.sr_step))
        for name, (g, Eg) in grads.items():
            self.W[name] = ops.update_weights(self.W[name], g, Eg, lr_m, lr_j, sr(name))
        for name, terms in sums.items():
            gc, Eg = ops.scalar_gradient(terms)
            T[name + ".gs"], T[name + ".Egs"] = gc, Eg
            self.scal[name] = ops.update_scalar(self.scal[name], gc, Eg, lr_m, lr_j, sr(name))
        self.sr_step += 1

    # ------------------------------------------------------------------ whole steps
    def block_step(self, a, e0, E0, lr_m, lr_j):
        """A lone residual block: int8 input, int8 error at its output."""
        self.trace = {}
        y = self.forward_blocks(a)
        grads, sums = {}, {}
        e, E = self.backward_blocks(e0, E0, grads, sums)
        self.apply_updates(grads, sums, lr_m, lr_j)
        return y, e, E

    def step(self, x_f32, labels, lr_m, lr_j):
        self.trace = T = {}
        y, gap = self.forward(x_f32)
        hw = self.out_hw * self.out_hw
        loss, d32, dW, db, logits = ops.head(gap, self.Wfc, self.bfc, labels, hw)
        T["head.logits"], T["head.d"] = logits, d32
        codes, E = sq_real(d32)
        e = np.broadcast_to(codes.astype(np.int8)[:, None, None, :], y.shape).copy()
        T["head.e"], T["head.E"] = e, E
        grads, sums = {}, {}
        e, E = self.backward_blocks(e, E, grads, sums)
        self.backward_stem(e, E, grads, sums)
        self.apply_updates(grads, sums, lr_m, lr_j)
        lr = float(lr_m) * 2.0 ** (-int(lr_j))
        self.Wfc = self.Wfc - lr * dW
        self.bfc = self.bfc - lr * db
        return loss
