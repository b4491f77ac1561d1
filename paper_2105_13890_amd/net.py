"""Sequencing of libeoq calls into whole full-int8 training steps of a Fixup residual network.

This module only decides WHICH C-ABI call runs on WHICH buffer; all arithmetic happens in the
library's kernels.  Layer arithmetic: Eq.2 (forward), Eq.3 (errors), Eq.4 (parameter gradients),
Eq.8-13 (quantisation strategies, update); block topology: the Fixup residual block of Section 3.1
(one multiplier per block, a bias before every convolution and every ReLU, a strided 1x1
convolution on the biased block input when the shape changes).  Everything a step needs stays
on the device: exponents, abs-max statistics, scalar-gradient sums and the learning rate live in
device slots, so a step enqueues kernels without a single host synchronisation and can be
captured into a HIP graph.

The backward pass runs on two HIP streams of equal priority: the error chain (ReLU backward, Q_e,
backward-data convolution, block merges) on the main stream, and each layer's parameter chain
(weight-gradient convolution, Q_g, update) on a side stream, joined by events: the parameter chain
of layer l starts when e3 of layer l exists, its update waits until the backward-data convolution has
read the old weights, and an error buffer that the side stream still reads is not handed out again
before that read has finished.  The two chains share no scratch memory.
"""
from __future__ import annotations

import zlib
from collections import deque
from dataclasses import dataclass, field

import numpy as np
import torch

import seeded_inputs as si

from . import eoq, fixup_init


@dataclass
class Unit:
    """One Fixup layer (Eq.2) and the buffers it owns."""
    name: str
    desc: eoq.ConvDesc
    b_pre: str | None
    gamma: str | None
    b_post: str | None
    relu: bool = True
    w: torch.Tensor = None            # int8 KRSC
    wt: torch.Tensor = None           # the same filters as CRSK (operand of the backward-data convolution)
    u: torch.Tensor = None            # int8 biased input x1 (what the convolution reads)
    mask: torch.Tensor = None         # ReLU bits
    t: torch.Tensor = None            # wide Q_a1 output (multiplier layers, shortcut convolutions)
    y: torch.Tensor = None            # int8 output, kept only where a later block adds it back

    @property
    def out_shape(self):
        d = self.desc
        return (d.N, d.P, d.Q, d.K)

    @property
    def in_shape(self):
        d = self.desc
        return (d.N, d.H, d.W, d.C)


@dataclass
class Block:
    name: str
    units: list
    ds: Unit | None


class _Slots:
    """Named int32 / int64 device slots (exponents, abs-max values, sums)."""

    def __init__(self):
        self.names32: dict[str, int] = {}
        self.names64: dict[str, int] = {}

    def i32(self, name):
        return self.names32.setdefault(name, len(self.names32))

    def i64(self, name):
        return self.names64.setdefault(name, len(self.names64))


class FixupNet:
    N_EBUF = 6     # rotating error buffers (at least 5: e1, e3, e4 of a layer, the shortcut error, the other merge input)

    def __init__(self, cfg: dict, batch: int, seed: int = 0, trace: bool = False, overlap: bool = True,
                 weights: dict | None = None, classifier=None, sr_seed: int | None = None):
        """weights: {layer name: int8 K x R x S x C codes} and classifier = (W fp64 [classes x features], b fp64):
        the initial parameters as input data.  Left out, they are drawn by fixup_init from `seed` and coded with
        Q_w by the library.  sr_seed: switch the update to the library's optional stochastic rounding (not the
        paper's rule; off by default), with this seed."""
        assert torch.cuda.is_available(), "libeoq needs the GPU; there is no CPU path"
        self.cfg, self.N, self.seed, self.tracing = dict(cfg), batch, seed, trace
        self.dev = torch.device("cuda")
        self.ctx = eoq.Context()
        self.overlap = overlap
        self.main = torch.cuda.current_stream()
        self.side = torch.cuda.Stream()            # default priority
        self.ctx_w = eoq.Context(self.side)        # parameter chain: dW, Q_g, update
        self._pending: dict[int, int] = {}      # error buffer -> index (in _side_ev) of the side stream's last read of it
        self._side_ev: list = []                # this step's events on the side stream, in the order they were recorded
        self._synced = -1                       # the main stream has waited for _side_ev[: _synced + 1]
        self._last_gdone = None                 # event after the latest multiplier-gradient sum of this step
        self._deferred = None                   # (layer, weight-gradient sums) whose update has not been enqueued yet
        self.ev_fwd = [torch.cuda.Event(), torch.cuda.Event()]      # fork / join of the two forward half-batch chains
        self.trace: dict[str, object] = {}
        self.prof = None                   # list of (kind, unit, work, start event, end event) while profiling
        bt = cfg["block"]
        N = batch
        hw, ch = cfg["in_hw"], cfg["in_ch"]
        self.scal_names: list[str] = []
        self.units: list[Unit] = []

        def D(h, c, k, r, st, pad):
            return eoq.ConvDesc(N, h, h, c, k, r, r, st, pad)

        self.stem = None
        self.pool = False
        if cfg["stem"] == "cifar":
            w0 = cfg["widths"][0]
            self.stem = Unit("stem", D(hw, ch, w0, 3, 1, 1), None, None, "stem.b")
            ch = w0
        elif cfg["stem"] == "imagenet":
            w0 = cfg["widths"][0]
            self.stem = Unit("stem", D(hw, ch, w0, 7, 2, 3), None, None, "stem.b")
            self.pool = True
            self.pool_in_hw = self.stem.desc.P
            hw = (self.pool_in_hw + 2 - 3) // 2 + 1
            ch = w0
        self.blocks: list[Block] = []
        for s_i, (depth, width) in enumerate(zip(cfg["depths"], cfg["widths"])):
            for b_i in range(depth):
                stride = 2 if (b_i == 0 and s_i > 0) else 1
                out_ch = width if bt == "basic" else 4 * width
                nm = f"s{s_i}b{b_i}"
                if bt == "basic":
                    c1 = Unit(nm + ".c1", D(hw, ch, width, 3, stride, 1), nm + ".b1a", None, nm + ".b1b")
                    c2 = Unit(nm + ".c2", D(c1.desc.P, width, width, 3, 1, 1), nm + ".b2a", nm + ".g", nm + ".b2b")
                    units = [c1, c2]
                else:
                    c1 = Unit(nm + ".c1", D(hw, ch, width, 1, 1, 0), nm + ".b1a", None, nm + ".b1b")
                    c2 = Unit(nm + ".c2", D(hw, width, width, 3, stride, 1), nm + ".b2a", None, nm + ".b2b")
                    c3 = Unit(nm + ".c3", D(c2.desc.P, width, out_ch, 1, 1, 0), nm + ".b3a", nm + ".g", nm + ".b3b")
                    units = [c1, c2, c3]
                ds = None
                if stride != 1 or ch != out_ch:
                    ds = Unit(nm + ".ds", D(hw, ch, out_ch, 1, stride, 0), None, None, None, relu=False)
                self.blocks.append(Block(nm, units, ds))
                hw, ch = units[-1].desc.P, out_ch
        self.out_hw, self.out_ch = hw, ch
        self.classes = cfg["classes"]

        # ---- parameters ------------------------------------------------------------------------
        all_units = ([self.stem] if self.stem else []) + [u for b in self.blocks for u in b.units + ([b.ds] if b.ds else [])]
        self.all_units = all_units
        for u in all_units:
            for s in (u.b_pre, u.gamma, u.b_post):
                if s and s not in self.scal_names:
                    self.scal_names.append(s)
        self.scal_idx = {n: i for i, n in enumerate(self.scal_names)}
        init = np.array([128 if n.endswith(".g") else 0 for n in self.scal_names] + [0], dtype=np.int32)
        self.scal = torch.from_numpy(init).to(self.dev)            # multiplier = 1 (code 128), biases = 0
        branch = {u.name for b in self.blocks for u in b.units}
        coeff = fixup_init.branch_coefficient(int(sum(cfg["depths"])), 2 if bt == "basic" else 3)
        for u in all_units:
            d = u.desc
            shape = (d.K, d.R, d.S, d.C)
            if weights is not None:
                w0 = np.ascontiguousarray(weights[u.name])
                assert w0.dtype == np.int8 and w0.shape == shape, (u.name, w0.dtype, w0.shape)
                u.w = torch.from_numpy(w0).to(self.dev)
            else:
                wf = torch.from_numpy(fixup_init.conv_weights_f32(seed, u.name, shape,
                                                                  coeff if u.name in branch else 1.0)).to(self.dev)
                u.w = torch.empty(shape, dtype=torch.int8, device=self.dev)
                self.ctx.quantize(wf, eoq.CQ, 0, u.w)              # Q_w = CQ (Eq.8)
            if d.C % 16 == 0 and d.K % 16 == 0:
                u.wt = torch.empty_like(u.w)                       # refreshed after every update, off the critical path
                self.ctx.transpose_filters(d, u.w, u.wt)
        if self.classes:
            Wc, bc = classifier if classifier is not None else fixup_init.classifier_f64(seed, self.classes, ch)
            self.Wfc = torch.from_numpy(np.ascontiguousarray(Wc, dtype=np.float64)).to(self.dev)
            self.bfc = torch.from_numpy(np.ascontiguousarray(bc, dtype=np.float64)).to(self.dev)
            assert self.Wfc.shape == (self.classes, ch) and self.bfc.shape == (self.classes,)

        # ---- buffers ---------------------------------------------------------------------------
        i8 = lambda shape: torch.empty(shape, dtype=torch.int8, device=self.dev)
        i32 = lambda shape: torch.empty(shape, dtype=torch.int32, device=self.dev)
        for u in all_units:
            n_out = int(np.prod(u.out_shape))
            if u.relu:
                u.mask = i32(((n_out + 31) // 32,))
            if not u.relu:
                # shortcut convolution: its output is read once more, as the wide skip input of the block's last
                # layer.  |t| <= 127^2 * R*S*C / 128 fits 16 bits for R*S*C <= 260, which halves that traffic.
                d = u.desc
                narrow = 127 * 127 * d.R * d.S * d.C // 128 + 1 < 2 ** 15
                u.t = torch.empty(u.out_shape, dtype=torch.int16 if narrow else torch.int32, device=self.dev)
            elif u.gamma and trace:
                u.t = i32(u.out_shape)       # multiplier layers: x2 is recomputed in the backward pass, stored only for inspection
        if self.stem:
            self.a0 = i8(self.stem.in_shape)
            self.stem.u = self.a0
            if self.pool:
                self.prepool = i8(self.stem.out_shape)
                self.pool_arg = torch.empty(self.blocks_in_shape(cfg, N), dtype=torch.uint8, device=self.dev)
                self.pool_spec = torch.full((1,), -1, dtype=torch.int32, device=self.dev)     # exponent of the pool's error, step to step
        for bi, b in enumerate(self.blocks):
            b.units[0].u = i8(b.units[0].in_shape)
            if b.ds:
                b.ds.u = b.units[0].u
            for u in b.units[1:]:
                u.u = i8(u.in_shape)
            b.a_in = None if b.ds else i8(b.units[0].in_shape)       # block input kept only as an identity shortcut
        self.y_out = i8(self.blocks[-1].units[-1].out_shape)
        max_act = max(max(int(np.prod(u.out_shape)), int(np.prod(u.in_shape))) for u in all_units)
        max_w = max(u.w.numel() for u in all_units)
        # few rotating error buffers: a buffer that was written a moment ago is still in the memory-side cache when
        # the next kernel reads it (one buffer per acquisition, which would spare the main stream every wait for
        # the side stream's reads, measured 10 % slower)
        self.ebuf = [i8((max_act,)) for _ in range(self.N_EBUF)]
        self.gacc = i32((max_w,))
        self.gq = i8((max_w,))
        ws_bytes = 16
        for u in all_units:
            for op in (eoq.OP_CONV_FWD, eoq.OP_CONV_BWD_DATA, eoq.OP_CONV_BWD_WEIGHT):
                ws_bytes = max(ws_bytes, eoq.Context.workspace_bytes(u.desc, op))
        self.ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=self.dev)
        self.ws_w = torch.empty((ws_bytes,), dtype=torch.uint8, device=self.dev)     # the side stream's own scratch
        for u in all_units:
            u.ev_e3, u.ev_dx, u.ev_done = (torch.cuda.Event() for _ in range(3))
            # exponent of this layer's backward-data sums in the previous step (what the next step tries first)
            u.spec = torch.full((1,), -1, dtype=torch.int32, device=self.dev)
        # ---- slots -------------------------------------------------------------------------------
        self.sl = _Slots()
        self._plan_slots()
        self.slots32 = torch.zeros((len(self.sl.names32) + 4,), dtype=torch.int32, device=self.dev)
        self.sums64 = torch.zeros((len(self.sl.names64) + 4,), dtype=torch.int64, device=self.dev)
        self.lr = torch.zeros((2,), dtype=torch.int32, device=self.dev)
        self.sgrad_tab = eoq.scalar_grad_table(self.sgrad_entries, self.dev)
        # optional stochastic rounding: {seed, step} on the device; a tensor's id in the hash is the CRC-32 of its name
        self.sr = None
        if sr_seed is not None:
            self.sr = torch.tensor([sr_seed & 0xFFFFFFFF, 0], dtype=torch.int64).to(torch.int32).to(self.dev)
            ids = np.array([zlib.crc32(p.encode("utf-8")) & 0xFFFFFFFF for p in self.sgrad_params], dtype=np.uint32)
            self.sr_scal_ids = torch.from_numpy(ids.view(np.int32).copy()).to(self.dev)
        self.g_code = i32((len(self.sgrad_entries) + 1,))
        self.g_exp = i32((len(self.sgrad_entries) + 1,))
        if self.classes:
            F, J = self.out_ch, self.classes
            self.gap = i32((N, F))
            self.loss = torch.zeros((1,), dtype=torch.float64, device=self.dev)
            self.d32 = torch.empty((N, F), dtype=torch.float32, device=self.dev)
            self.logits = torch.empty((N, J), dtype=torch.float64, device=self.dev)
            self.head_codes = i8((N, F))
            self.head_ws = torch.empty((eoq.Context.head_workspace_bytes(N, F, J) // 8 + 1,), dtype=torch.float64,
                                       device=self.dev)
            self.x_in = torch.empty(self.stem.in_shape, dtype=torch.float32, device=self.dev)
            self.labels = torch.zeros((N,), dtype=torch.int32, device=self.dev)
        torch.cuda.synchronize()

    # ------------------------------------------------------------------------------------------
    def _plan_slots(self):
        """Name every device slot once and build the scalar-gradient table (Eq.4 for scalars)."""
        sl = self.sl
        entries: dict[str, list] = {}

        def term(param, sum_name, exp_name, off):
            entries.setdefault(param, []).append((sl.i64(sum_name), sl.i32(exp_name), off))

        if self.classes:
            e_name = "head.E"
        else:
            e_name = "ext.E"
        sl.i32(e_name)
        self.E_top = e_name
        for b in reversed(self.blocks):
            E0 = e_name
            for i in range(len(b.units) - 1, -1, -1):
                u = b.units[i]
                u.E0 = e_name
                term(u.b_post, u.name + ".S_e1", e_name, 0)
                if u.gamma:
                    term(u.gamma, u.name + ".S_e1t", e_name, -7)
                    u.E3 = u.name + ".E3"
                else:
                    u.E3 = e_name
                u.E4 = u.name + ".E4"
                term(u.b_pre, u.name + ".S_e4", u.E4, 0)
                for nm in (u.E3, u.E4, u.name + ".Eg", u.name + ".M_e1", u.name + ".M_D", u.name + ".M_G",
                           u.name + ".gmax"):
                    sl.i32(nm)
                e_name = u.E4
            if b.ds:
                d = b.ds
                d.E0 = d.E3 = E0
                d.E4 = d.name + ".E4"
                term(b.units[0].b_pre, d.name + ".S_e4", d.E4, 0)
                for nm in (d.E4, d.name + ".Eg", d.name + ".M_D", d.name + ".M_G", d.name + ".gmax"):
                    sl.i32(nm)
            sl.i32(b.name + ".M_in")
            sl.i32(b.name + ".M_inm")
            e_name = b.name + ".E_in"
            sl.i32(e_name)
        if self.stem:
            s = self.stem
            if self.pool:
                sl.i32("pool.M")
                sl.i32("pool.E")
                e_name = "pool.E"
            s.E0 = s.E3 = e_name
            term(s.b_post, s.name + ".S_e1", e_name, 0)
            for nm in (s.name + ".Eg", s.name + ".M_e1", s.name + ".M_G", s.name + ".gmax"):
                sl.i32(nm)
        self.sgrad_params = list(entries.keys())
        self.sgrad_entries = [(self.scal_idx[p], entries[p]) for p in self.sgrad_params]

    @staticmethod
    def blocks_in_shape(cfg, N):
        """Shape of the pooled stem output (ImageNet-shaped stem: conv 7x7/2 then pool 3x3/2)."""
        h = (cfg["in_hw"] + 6 - 7) // 2 + 1
        h = (h + 2 - 3) // 2 + 1
        return (N, h, h, cfg["widths"][0])

    def s32(self, name):
        i = self.sl.names32[name]
        return self.slots32[i:i + 1]

    def s64(self, name):
        i = self.sl.names64[name]
        return self.sums64[i:i + 1]

    def sc(self, name):
        if name is None:
            return None
        i = self.scal_idx[name]
        return self.scal[i:i + 1]

    def _call(self, kind, unit, work, fn, *args, stream=None, **kw):
        """Run one library call; when profiling, bracket it with events on the stream it is enqueued on."""
        if self.prof is None:
            return fn(*args, **kw)
        stream = stream or self.main
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        r = fn(*args, **kw)
        e1.record(stream)
        self.prof.append((kind, unit, work, e0, e1))
        return r

    def _rec(self, name, t):
        if self.tracing:
            if self.overlap:
                torch.cuda.synchronize()      # inspection only: the copy below runs on the main stream
            self.trace[name] = t.detach().clone()

    def _acquire(self, bufs):
        """Next free error buffer; if the side stream may still read its previous content, the main stream waits for
        that read (waiting for a later event of the side stream instead, to cover the buffers acquired next with
        one wait, stalls the main stream whenever the side stream runs a layer or two behind: measured slower)."""
        b = bufs.popleft()
        k = self._pending.pop(b.data_ptr(), -1)
        if k > self._synced:
            self.main.wait_event(self._side_ev[k])
            self._synced = k
        return b

    def set_lr(self, m: int, j: int):
        self.lr.copy_(torch.tensor([m, j], dtype=torch.int32))

    @staticmethod
    def _conv_work(u):
        d = u.desc
        return 2.0 * d.N * d.P * d.Q * d.K * d.C * d.R * d.S       # algorithmic ops (multiply-add = 2)

    # ------------------------------------------------------------------------------------------ forward
    def _unit_fwd(self, u: Unit, skip=None, y=None, u_next=None, b_next=None, side=False, half=None, src=None,
                  keep=True):
        """One forward convolution with its fused epilogue (Eq.2).  half = 0 / 1: only that half of the batch (every
        tensor is batch-major, so a half is a contiguous slice), on the main / side stream.  src: the biased input to
        read instead of the layer's own stored copy; keep = False (inference): no ReLU mask is written."""
        side = side or half == 1
        c, ws, st = (self.ctx_w, self.ws_w, self.side) if side else (self.ctx, self.ws, self.main)
        x1 = u.u if src is None else src
        desc, sl = u.desc, (lambda t: t)
        if half is not None:
            d = u.desc
            desc = eoq.ConvDesc(d.N // 2, d.H, d.W, d.C, d.K, d.R, d.S, d.stride, d.pad)

            def sl(t):
                if t is None:
                    return None
                n = t.numel() // 2
                return t.view(-1)[half * n:(half + 1) * n]
        if not u.relu:
            ep = c.epilogue(relu=0, t_wide=sl(u.t))
        else:
            ep = c.epilogue(gamma=self.sc(u.gamma), b_post=self.sc(u.b_post), skip=sl(skip), relu=1,
                            b_next_pre=self.sc(b_next), y=sl(y), u_next=sl(u_next), mask=sl(u.mask) if keep else None,
                            t_wide=sl(u.t) if keep else None)
        self._call("conv_fwd", u.name, self._conv_work(u), c.conv_fwd, desc, sl(x1), u.w, ep=ep, ws=ws, stream=st)
        if self.tracing:
            self._rec(u.name + ".u", u.u)
            if u.t is not None:
                self._rec(u.name + ".t", u.t)
            if u.relu:
                self._rec(u.name + ".mask", u.mask)
                if y is not None:
                    self._rec(u.name + ".y", y)

    def _can_split_forward(self):
        """Nothing in the forward pass of the blocks looks across images, so the two halves of the batch can run as
        two independent chains.  Needs an even batch and mask words that do not straddle the halves."""
        return (self.overlap and not self.tracing and self.N % 2 == 0 and
                all(int(np.prod(u.out_shape)) % 64 == 0 for b in self.blocks for u in b.units))

    def _forward_blocks(self):
        if self._can_split_forward():
            # two half-batch chains, one per stream: a convolution of this size leaves the chip partly idle while it
            # starts and drains, and a chain of dependent launches cannot hide that; two independent chains can
            self.ev_fwd[0].record(self.main)
            self.side.wait_event(self.ev_fwd[0])
            for bi, b in enumerate(self.blocks):
                nxt = self.blocks[bi + 1] if bi + 1 < len(self.blocks) else None
                for half in (0, 1):
                    self._forward_block(b, nxt, half)
            self.ev_fwd[1].record(self.side)
            self.main.wait_event(self.ev_fwd[1])
            return
        for bi, b in enumerate(self.blocks):
            self._forward_block(b, self.blocks[bi + 1] if bi + 1 < len(self.blocks) else None, None)

    def _forward_block(self, b, nxt, half):
        fork = b.ds is not None and self.overlap and half is None
        if b.ds:
            # whole-batch chain: the shortcut convolution only meets the branch at the block's last layer, so it runs
            # beside the branch on the side stream (it is bound by its wide stores, the branch's first layers are not)
            if fork:
                b.ds.ev_e3.record(self.main)
                self.side.wait_event(b.ds.ev_e3)
            self._unit_fwd(b.ds, side=fork, half=half)
            if fork:
                b.ds.ev_dx.record(self.side)
        for i, u in enumerate(b.units):
            last = i == len(b.units) - 1
            if not last:
                n_u = b.units[i + 1]
                self._unit_fwd(u, u_next=n_u.u, b_next=n_u.b_pre, y=self._dbg_y(u), half=half)
            else:
                if fork:
                    self.main.wait_event(b.ds.ev_dx)
                skip = b.ds.t if b.ds else b.a_in
                if nxt is not None:
                    self._unit_fwd(u, skip=skip, y=nxt.a_in if nxt.a_in is not None else self._dbg_y(u),
                                   u_next=nxt.units[0].u, b_next=nxt.units[0].b_pre, half=half)
                else:
                    self._unit_fwd(u, skip=skip, y=self.y_out, half=half)

    def _dbg_y(self, u):
        """Unbiased int8 output of an inner layer: only materialised when tracing (tests compare it)."""
        if not self.tracing:
            return None
        return torch.empty(u.out_shape, dtype=torch.int8, device=self.dev)

    def forward(self):
        """x_in (fp32 NHWC) -> Q input, stem, (pool), blocks, pooled integer sums."""
        c = self.ctx
        b0 = self.blocks[0]
        # network input: CQ(x / 4); a streaming pass, 4 B in + 1 B out per element
        self._call("hbm_quantize", "input", 5.0 * self.x_in.numel(), c.quantize, self.x_in, eoq.CQ, -2, self.a0)
        self._rec("in.a", self.a0)
        s = self.stem
        if self.pool:
            self._unit_fwd(s, y=self.prepool)
            self._rec("stem.prepool", self.prepool)
            d = s.desc
            yb = b0.a_in if b0.a_in is not None else (torch.empty(b0.units[0].in_shape, dtype=torch.int8, device=self.dev)
                                                      if self.tracing else None)
            c.maxpool_fwd(self.prepool, d.N, d.P, d.Q, d.K, 3, 3, 2, 1, yb, self.sc(b0.units[0].b_pre), b0.units[0].u,
                          self.pool_arg)
            if yb is not None:
                self._rec("pool.y", yb)
        else:
            self._unit_fwd(s, y=b0.a_in if b0.a_in is not None else self._dbg_y(s), u_next=b0.units[0].u,
                           b_next=b0.units[0].b_pre)
        self._forward_blocks()
        hw = self.out_hw * self.out_hw
        c.gap_sum(self.y_out, self.N, hw, self.out_ch, self.gap)
        self._rec("gap.sum", self.gap)

    # ------------------------------------------------------------------------------------------ inference
    def forward_inference(self):
        """The int8 forward chain on its own (Eq.2 layer by layer, no BatchNorm anywhere): x_in -> pooled integer
        sums, the same kernels as the training forward with every training side output switched off -- no ReLU masks,
        no stored per-layer inputs, no pool winners.  Activations live in a few rotating buffers (the backward
        pass's scratch buffers, idle here); the only wide tensor is a shape-changing block's shortcut, consumed by
        that block's last layer.  Two half-batch chains as in training."""
        c = self.ctx
        b0 = self.blocks[0]
        free = deque(self.ebuf)

        def buf(shape):
            t = free.popleft()
            free.append(t)
            return t[:int(np.prod(shape))].view(shape)

        c.quantize(self.x_in, eoq.CQ, -2, self.a0)
        s = self.stem
        first_in = b0.units[0].in_shape
        u_cur = buf(first_in)                                    # biased input of the first block
        y_cur = buf(first_in) if b0.ds is None else None         # unbiased copy, only where an identity shortcut adds it
        if self.pool:
            d = s.desc
            self._unit_fwd(s, y=self.prepool, keep=False)
            c.maxpool_fwd(self.prepool, d.N, d.P, d.Q, d.K, 3, 3, 2, 1, y_cur, self.sc(b0.units[0].b_pre), u_cur, None)
        else:
            self._unit_fwd(s, y=y_cur, u_next=u_cur, b_next=b0.units[0].b_pre, keep=False)
        split = self._can_split_forward()
        if split:
            self.ev_fwd[0].record(self.main)
            self.side.wait_event(self.ev_fwd[0])
        for bi, b in enumerate(self.blocks):
            nxt = self.blocks[bi + 1] if bi + 1 < len(self.blocks) else None
            out_shape = b.units[-1].out_shape
            inner = [buf(u.in_shape) for u in b.units[1:]]
            if nxt is not None:
                u_out = buf(out_shape)
                y_out = buf(out_shape) if nxt.ds is None else None
            else:
                u_out, y_out = None, self.y_out
            for half in ((0, 1) if split else (None,)):
                if b.ds:
                    self._unit_fwd(b.ds, half=half, src=u_cur)            # wide shortcut: the block's only stored extra
                x = u_cur
                for i, u in enumerate(b.units[:-1]):
                    self._unit_fwd(u, u_next=inner[i], b_next=b.units[i + 1].b_pre, half=half, src=x, keep=False)
                    x = inner[i]
                skip = b.ds.t if b.ds else y_cur
                self._unit_fwd(b.units[-1], skip=skip, y=y_out, u_next=u_out,
                               b_next=nxt.units[0].b_pre if nxt is not None else None, half=half, src=x, keep=False)
            u_cur, y_cur = u_out, y_out
        if split:
            self.ev_fwd[1].record(self.side)
            self.main.wait_event(self.ev_fwd[1])
        c.gap_sum(self.y_out, self.N, self.out_hw * self.out_hw, self.out_ch, self.gap)

    # ------------------------------------------------------------------------------------------ backward
    def _grad(self, u: Unit, e3, e3_buf, gamma_e1=None):
        """Weight-gradient sums e3 * x1 (Eq.4) on the side stream once e3 exists; Q_g (Eq.12) and the update follow in
        _apply_update.  A wait for an event of another stream costs the waiting stream several microseconds even
        when the event has long happened, so the side stream waits ONCE per layer, here, and everything else it
        needs is ordered through that wait: the main stream produced e3 after the backward-data call of the layer
        above, so that layer's update (deferred until now) may overwrite its weights; e1 exists before e3, so the
        multiplier-gradient sum of this layer (gamma_e1: its e1 buffer) is enqueued here too."""
        if not self.overlap:
            if gamma_e1 is not None:
                self._gamma_sum(u, gamma_e1, self.ctx, self.main)
            G = self.gacc[:u.w.numel()]
            self._call("conv_bwd_weight", u.name, self._conv_work(u), self.ctx.conv_bwd_weight, u.desc, e3, u.u, G,
                       self.s32(u.name + ".M_G"), self.ws, stream=self.main)
            return G
        u.ev_e3.record(self.main)
        self.side.wait_event(u.ev_e3)
        self._flush_update()
        if gamma_e1 is not None:
            self._gamma_sum(u, gamma_e1, self.ctx_w, self.side)
        G = self.gacc[:u.w.numel()]
        self._call("conv_bwd_weight", u.name, self._conv_work(u), self.ctx_w.conv_bwd_weight, u.desc, e3, u.u, G,
                   self.s32(u.name + ".M_G"), self.ws_w, stream=self.side)
        u.ev_done.record(self.side)
        self._side_ev.append(u.ev_done)
        k = len(self._side_ev) - 1
        self._pending[e3_buf.data_ptr()] = k               # neither e3 nor e1 is overwritten before the side stream
        if gamma_e1 is not None:                           # has read it
            self._pending[gamma_e1.data_ptr()] = k
            self._last_gdone = k
        return G

    def _flush_update(self, final=False):
        """Apply the deferred update.  final: no later layer orders it behind the backward-data call that read the
        old weights, so the side stream waits for the main stream as it stands."""
        if self._deferred is None:
            return
        u, G = self._deferred
        self._deferred = None
        if final and self.overlap:
            u.ev_dx.record(self.main)
            self.side.wait_event(u.ev_dx)
        self._apply_update(u, G)

    def _apply_update(self, u: Unit, G):
        """g_w = Q_g(G) (Eq.12), W <- Q_w(W - Q_u(lr g_w)) (Eq.13), and the transposed copy the next backward-data
        call multiplies with: one fused call; three separate ones when tracing, which records the gradient codes."""
        c = self.ctx_w if self.overlap else self.ctx
        M_G, Eg, gmax = self.s32(u.name + ".M_G"), self.s32(u.name + ".Eg"), self.s32(u.name + ".gmax")
        if not self.tracing:
            n = u.w.numel()
            self._call("hbm_grad_update", u.name, (4 + 1 + (2 if u.wt is not None else 1)) * float(n), c.grad_update, u.desc,
                       G, M_G, self.s32(u.E3), -7, self.lr, u.w, wt=u.wt, exp_out=Eg, max_code_out=gmax,
                       sr_slot=self.sr, tensor_id=self._tid(u.name), stream=self.side if self.overlap else self.main)
            return
        n = u.w.numel()
        g = self.gq[:n]
        c.requant_epilogue(eoq.RQ_SQ_ACC, n, acc=G, absmax=M_G, exp_in=self.s32(u.E3), exp_in_off=-7, out=g,
                           exp_out=Eg, max_code_out=gmax)
        self._rec(u.name + ".G", G.view(u.w.shape))
        self._rec(u.name + ".gw", g.view(u.w.shape))
        c.update_int8(u.w, g, Eg, gmax, self.lr, sr_slot=self.sr, tensor_id=self._tid(u.name))
        if u.wt is not None:
            c.transpose_filters(u.desc, u.w, u.wt)

    @staticmethod
    def _tid(name: str) -> int:
        return zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF

    def _gamma_sum(self, u: Unit, e1, c, st):
        """Sum of e1 * x2 for the multiplier's gradient (Eq.4), with x2 recomputed from (u, w) instead of having
        been stored by the forward pass.  Nothing on the error chain waits for it -- only the scalar update at the
        end of the step does -- so the convolution runs on the side stream."""
        n_out = int(np.prod(u.out_shape))
        self._call("relu_bwd_recompute", u.name, self._conv_work(u), c.relu_bwd_recompute, u.desc, u.u, u.w,
                   e1[:n_out], None, None, None, self.s64(u.name + ".S_e1t"), None, stream=st)

    def _unit_bwd(self, u: Unit, e0, bufs, need_dx=True, relu_done=False, fuse_below: Unit | None = None,
                  merge=None, e3_done=None):
        """Eq.3 / Eq.4 for one layer; e0 is overwritten by e1.  Returns (buffer with the error for the layer
        below or None, e1).  relu_done: e0 already is e1 (the ReLU backward step was fused into the call that
        produced it).  fuse_below: the layer whose output is this layer's input -- its ReLU backward step and
        sums are applied by this layer's backward-data call, which then returns e1 of that layer instead of e4.
        merge = (other error buffer, its exponent slot, abs-max slot): this layer's e4 is one of the two errors
        that meet at the block input; the statistics of their sum are taken by the same call (a fourth and fifth
        entry: the mask of the layer receiving the merged error and the slot for the maximum under that mask).
        e3_done: buffer that already holds Q_e(e1 * gamma) (written by the merge pass that produced e1)."""
        c = self.ctx
        n_out = int(np.prod(u.out_shape))
        e1 = e0
        if u.relu and not relu_done:
            c.relu_bwd(e0[:n_out], u.mask, None, e1[:n_out], self.s64(u.name + ".S_e1"), None,
                       self.s32(u.name + ".M_e1"))
        if u.gamma and e3_done is not None:
            e3 = e3_done
        elif u.gamma:
            e3 = self._acquire(bufs)
            c.requant_epilogue(eoq.RQ_SQ_GAMMA, n_out, src_a=e1[:n_out], gamma=self.sc(u.gamma),
                               absmax=self.s32(u.name + ".M_e1"), exp_in=self.s32(u.E0), out=e3[:n_out],
                               exp_out=self.s32(u.E3))
        else:
            e3 = e1
        if self.tracing:
            self._rec(u.name + ".e3", e3[:n_out].view(u.out_shape))
        g = self._grad(u, e3[:n_out], e3, gamma_e1=e1 if (u.relu and u.gamma) else None)
        e4 = None
        if need_dx:
            n_in = int(np.prod(u.in_shape))
            e4 = self._acquire(bufs)
            if fuse_below is not None:
                assert fuse_below.relu and not fuse_below.gamma and fuse_below.out_shape == u.in_shape
                e4_dbg = torch.empty(u.in_shape, dtype=torch.int8, device=self.dev) if self.tracing else None
                f = fuse_below
                self._call("conv_bwd_data", u.name, self._conv_work(u), c.conv_bwd_data_sq, u.desc, e3[:n_out], u.w,
                           e4_dbg, self.s32(u.name + ".M_D"), self.s32(u.E3), -7, self.s32(u.E4),
                           self.s64(u.name + ".S_e4"), self.ws, w_transposed=u.wt, mask=f.mask, e1=e4[:n_in],
                           spec_state=None if self.tracing else u.spec, sum_e1=self.s64(f.name + ".S_e1"),
                           absmax_e1=self.s32(f.name + ".M_e1") if self.tracing else None)   # only Q_e(e1*gamma) reads it
                if self.tracing:
                    self._rec(u.name + ".e4", e4_dbg)
            else:
                mg = {}
                if merge is not None:
                    mg = dict(merge_other=merge[0][:n_in], merge_exp_other=self.s32(merge[1]),
                              merge_absmax=self.s32(merge[2]))
                    if len(merge) > 3:
                        mg.update(merge_mask=merge[3], merge_absmax_masked=self.s32(merge[4]))
                self._call("conv_bwd_data", u.name, self._conv_work(u), c.conv_bwd_data_sq, u.desc, e3[:n_out], u.w,
                           e4[:n_in], self.s32(u.name + ".M_D"), self.s32(u.E3), -7, self.s32(u.E4),
                           self.s64(u.name + ".S_e4"), self.ws, w_transposed=u.wt,
                           spec_state=None if self.tracing else u.spec, **mg)
                if self.tracing:
                    self._rec(u.name + ".e4", e4[:n_in].view(u.in_shape))
        # the update, once every reader of the old weights has run: behind the next layer's wait on the side stream
        if self.overlap and need_dx:
            self._deferred = (u, g)
        else:
            self._apply_update(u, g)
        if u.gamma:
            bufs.append(e3)
        return e4, e1

    def _backward_blocks(self, e, bufs):
        """e: buffer holding the error at the last block's output (exponent slot self.E_top)."""
        c = self.ctx
        masked = False                     # the error handed down already went through the receiving layer's ReLU
        e3_low = None                      # ... and Q_e(e1 * gamma) of that layer exists as well
        for bi in range(len(self.blocks) - 1, -1, -1):
            b = self.blocks[bi]
            assert len(b.units) >= 2
            last = b.units[-1]
            # the layer that receives this block's merged input error: the last layer of the block below.  Its ReLU
            # backward step (mask, bias-gradient sum) and its Q_e(e1 * gamma) ride on the merge pass
            low = self.blocks[bi - 1].units[-1] if bi > 0 and not self.tracing else None
            M_in, M_inm = b.name + ".M_in", b.name + ".M_inm"
            mstat = (low.mask, M_inm) if low is not None else ()
            # e now holds e1 of the last layer = shortcut error; its backward-data call already applies the ReLU
            # backward step of the layer below it, and so on down the branch
            e4, e_sk = self._unit_bwd(last, e, bufs, relu_done=masked,
                                      fuse_below=b.units[-2] if len(b.units) > 1 else None, e3_done=e3_low)
            E_sk = last.E0
            cur = e4
            for idx in range(len(b.units) - 2, -1, -1):
                # the first layer's e4 meets the shortcut error at the block input (identity shortcut: e_sk itself)
                mg = (e_sk, E_sk, M_in) + mstat if (idx == 0 and not b.ds) else None
                nxt, _ = self._unit_bwd(b.units[idx], cur, bufs, relu_done=True,
                                        fuse_below=b.units[idx - 1] if idx > 0 else None, merge=mg)
                bufs.append(cur)
                cur = nxt
            first = b.units[0]
            n_in = int(np.prod(first.in_shape))
            if b.ds:
                e4d, _ = self._unit_bwd(b.ds, e_sk, bufs, merge=(cur, first.E4, M_in) + mstat)
                other, E_other = e4d, b.ds.E4
            else:
                other, E_other = e_sk, E_sk
            out = cur
            extra = {}
            e3_low = None
            if low is not None:
                e3_low = self._acquire(bufs)
                extra = dict(mask=low.mask, sum_out=self.s64(low.name + ".S_e1"), gamma=self.sc(low.gamma),
                             out_b=e3_low[:n_in], exp_out_b=self.s32(low.E3), absmax_masked=self.s32(M_inm))
            # 2 B in + 1 B out per element (+ 1/8 B of mask and a second output byte when the next layer rides along)
            self._call("hbm_merge", b.name, (3 + (1.125 if low is not None else 0)) * float(n_in), c.requant_epilogue,
                       eoq.RQ_SQ_MERGE, n_in, src_a=cur[:n_in], src_b=other[:n_in], exp_in=self.s32(first.E4),
                       exp_b=self.s32(E_other), absmax=self.s32(M_in), out=out[:n_in],
                       exp_out=self.s32(b.name + ".E_in"), **extra)
            masked = low is not None
            if b.ds:
                bufs.append(e4d)
            bufs.append(e_sk)
            if self.tracing:
                self._rec(b.name + ".e_in", out[:n_in].view(first.in_shape))
            e = out
        return e

    def _backward_stem(self, e, bufs):
        c = self.ctx
        s = self.stem
        d = s.desc
        masked = False
        if self.overlap:
            # The side stream has nothing to do while the main stream runs the last merge and the pool's backward
            # pass: the float classifier's update goes there.  It is ordered behind the head's kernels through the
            # side stream's waits for the main stream since, and before the next step's head by the join.
            self.ctx_w.head_update(self.N, self.out_ch, self.classes, self.Wfc, self.bfc, self.lr, self.head_ws)
        if self.pool:
            n = int(np.prod(s.out_shape))
            e2 = self._acquire(bufs)
            # pool backward + Q_e; outside tracing also the stem's ReLU backward step (its mask, its bias-gradient sum)
            fuse = {} if self.tracing else dict(mask=s.mask, sum_out=self.s64(s.name + ".S_e1"),
                                                spec_state=self.pool_spec)
            c.maxpool_bwd_sq(self.pool_arg, e, d.N, d.P, d.Q, d.K, 3, 3, 2, 1, e2[:n], self.s32("pool.M"),
                             self.s32(self.blocks[0].name + ".E_in"), self.s32("pool.E"), **fuse)
            masked = not self.tracing
            bufs.append(e)
            e = e2
            if self.tracing:
                self._rec("pool.e", e[:n].view(s.out_shape))
        self._unit_bwd(s, e, bufs, need_dx=False, relu_done=masked)
        bufs.append(e)

    def _update_scalars(self):
        if self.overlap and self._last_gdone is not None and self._last_gdone > self._synced:
            self.main.wait_event(self._side_ev[self._last_gdone])       # the multiplier-gradient sums come from the side stream
            self._synced = self._last_gdone
        self.ctx.update_scalars(self.scal, self.sgrad_tab, len(self.sgrad_entries), self.sums64, self.slots32, self.lr,
                                self.g_code, self.g_exp, sr_slot=self.sr,
                                tensor_ids=self.sr_scal_ids if self.sr is not None else None)

    def _join(self):
        """End of a step: everything the side stream did is ordered before what the main stream does next."""
        self._flush_update(final=True)
        if self.overlap:
            self.main.wait_stream(self.side)
        self._pending.clear()
        self._side_ev.clear()
        self._synced = -1
        self._last_gdone = None

    # ------------------------------------------------------------------------------------------ whole steps
    def _zero_stats(self):
        self.ctx.fill_zero(self.slots32)
        self.ctx.fill_zero(self.sums64)

    def enqueue_step(self):
        """One full training step on the resident batch (x_in, labels): forward, head, backward, update.
        Only enqueues kernels; safe to capture into a HIP graph."""
        c = self.ctx
        self._zero_stats()
        self.forward()
        N, F, J = self.N, self.out_ch, self.classes
        hw = self.out_hw * self.out_hw
        # the classifier's own update feeds nothing in this step: with two streams it runs on the side stream at the
        # tail of the backward pass (see _backward_stem), not between the forward and the backward pass
        c.head_fwd_bwd(N, F, J, hw, self.gap, self.Wfc, self.bfc, self.labels, None if self.overlap else self.lr,
                       self.loss, self.d32, self.logits, self.head_ws)
        c.quantize(self.d32, eoq.SQ, 0, self.head_codes, self.s32("head.E"))     # Q_e on the head's error
        bufs = deque(self.ebuf)
        e = self._acquire(bufs)
        n_out = N * hw * F
        c.broadcast_hw(self.head_codes, N, hw, F, e[:n_out])
        if self.tracing:
            self._rec("head.logits", self.logits)
            self._rec("head.d", self.d32)
            self._rec("head.e", e[:n_out].view(self.blocks[-1].units[-1].out_shape))
        e = self._backward_blocks(e, bufs)
        self._backward_stem(e, bufs)
        self._update_scalars()
        self._join()
        if self.sr is not None:
            self.ctx.sr_next_step(self.sr)          # behind every update of this step, on both streams
        if self.tracing:
            self._rec("slots32", self.slots32)
            self._rec("g_code", self.g_code)
            self._rec("g_exp", self.g_exp)

    def capture_step(self) -> "torch.cuda.CUDAGraph":
        """Capture one training step (both streams) into a HIP graph; replaying it runs the step on whatever
        x_in / labels / lr hold at that time.  The network must have been built, and at least one step run
        eagerly, with a non-default stream current (the library's calls go to the stream that was current at
        construction, and the default stream cannot be captured); that same stream must be current now."""
        assert not self.tracing, "a traced step copies tensors out between calls and cannot be captured"
        assert self.main != torch.cuda.default_stream(), "build the network under torch.cuda.stream(<own stream>)"
        assert torch.cuda.current_stream() == self.main
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=self.main):
            self.enqueue_step()
        return g

    def step(self, x_f32: np.ndarray | torch.Tensor, labels, lr_m: int, lr_j: int) -> float:
        """Convenience wrapper: upload a batch, run one step, return the loss (synchronises)."""
        self.trace = {}
        xt = torch.as_tensor(x_f32)
        self.x_in.copy_(xt.to(self.dev, non_blocking=False))
        self.labels.copy_(torch.as_tensor(labels).to(self.dev))
        self.set_lr(lr_m, lr_j)
        self.enqueue_step()
        torch.cuda.synchronize()
        return float(self.loss.item())

    def block_step(self, a: np.ndarray, e0: np.ndarray, E0: int, lr_m: int, lr_j: int):
        """A lone residual block (no stem, no head): int8 input codes, int8 error at the output with exponent E0."""
        self.trace = {}
        c = self.ctx
        b0 = self.blocks[0]
        self.set_lr(lr_m, lr_j)
        self._zero_stats()
        at = torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        if b0.a_in is not None:
            b0.a_in.copy_(at)
        c.pre_bias(at, self.sc(b0.units[0].b_pre), b0.units[0].u)            # Eq.2 line x1
        self._forward_blocks()
        bufs = deque(self.ebuf)
        e = self._acquire(bufs)
        n = e0.size
        e[:n].copy_(torch.from_numpy(np.ascontiguousarray(e0)).to(self.dev).view(-1))
        self.s32(self.E_top).fill_(E0)
        e = self._backward_blocks(e, bufs)
        self._update_scalars()
        self._join()
        if self.sr is not None:
            self.ctx.sr_next_step(self.sr)
        if self.tracing:
            self._rec("slots32", self.slots32)
            self._rec("g_code", self.g_code)
            self._rec("g_exp", self.g_exp)
        torch.cuda.synchronize()
        n_in = int(np.prod(b0.units[0].in_shape))
        return self.y_out, e[:n_in].view(b0.units[0].in_shape)

    # ------------------------------------------------------------------------------------------ inspection
    def slot_value(self, name) -> int:
        return int(self.slots32[self.sl.names32[name]].item())

    def scalars(self) -> dict:
        v = self.scal.cpu().numpy()
        return {n: int(v[i]) for n, i in self.scal_idx.items()}

    def status(self) -> int:
        return self.ctx.status() | self.ctx_w.status()

    def spec_counters(self) -> tuple[int, int]:
        """(hits, misses) of the speculative backward-data / pool-backward calls since the network was built."""
        a, b = self.ctx.spec_counters(), self.ctx_w.spec_counters()
        return a[0] + b[0], a[1] + b[1]
