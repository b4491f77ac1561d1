"""GPU parity at the full sizes and in the launch configuration the benchmark times (ResNet-50 layers at
batch 128): the oracle cannot run whole tensors of that size in seconds, so sampled outputs are computed
one by one from the definitions (Eq.2 conv, Eq.3 e4, Eq.4 g_w), plus properties that hold at any size."""
import numpy as np
import pytest

import seeded_inputs as si

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle import ops as oo                    # noqa: E402
from oracle import quant as oq                  # noqa: E402
from oracle.ops import ConvShape                # noqa: E402
from oracle.net import Net as OracleNet         # noqa: E402

N = 128
LAYERS = [
    ("s0.c2", ConvShape(N, 56, 56, 64, 64, 3, 3, 1, 1)),
    ("s0.c3", ConvShape(N, 56, 56, 64, 256, 1, 1, 1, 0)),
    ("s1.ds", ConvShape(N, 56, 56, 256, 512, 1, 1, 2, 0)),
    ("s1.c2s", ConvShape(N, 56, 56, 128, 128, 3, 3, 2, 1)),
    ("s2.c2", ConvShape(N, 14, 14, 256, 256, 3, 3, 1, 1)),
    ("s3.c1", ConvShape(N, 7, 7, 2048, 512, 1, 1, 1, 0)),
]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def fwd_sample(d, u, w, n, p, q, k):
    s = 0
    for r in range(d.R):
        for t in range(d.S):
            h, x = p * d.stride + r - d.pad, q * d.stride + t - d.pad
            if 0 <= h < d.H and 0 <= x < d.W:
                s += int(np.dot(u[n, h, x].astype(np.int64), w[k, r, t].astype(np.int64)))
    return s


def dx_sample(d, e, w, n, h, x, c):
    s = 0
    for r in range(d.R):
        for t in range(d.S):
            ph, qw = h + d.pad - r, x + d.pad - t
            if ph < 0 or qw < 0 or ph % d.stride or qw % d.stride:
                continue
            p, q = ph // d.stride, qw // d.stride
            if p < d.P and q < d.Q:
                s += int(np.dot(e[n, p, q].astype(np.int64), w[:, r, t, c].astype(np.int64)))
    return s


def dw_sample(d, e, u, k, r, t, c):
    ps = np.arange(d.P)
    qs = np.arange(d.Q)
    hs, xs = ps * d.stride + r - d.pad, qs * d.stride + t - d.pad
    pv, qv = (hs >= 0) & (hs < d.H), (xs >= 0) & (xs < d.W)
    ee = e[:, ps[pv]][:, :, qs[qv], k].astype(np.int64)
    uu = u[:, hs[pv]][:, :, xs[qv], c].astype(np.int64)
    return int((ee * uu).sum())


@pytest.mark.parametrize("name,d", LAYERS, ids=[l[0] for l in LAYERS])
def test_resnet50_layer_calls_at_batch_128(name, d):
    from paper_2105_13890_amd import eoq
    ctx = eoq.Context()
    rng = np.random.default_rng(1)
    u = si.uniform_int8(11, name + ".u", (d.N, d.H, d.W, d.C))
    w = si.uniform_int8(11, name + ".w", (d.K, d.R, d.S, d.C), -40, 40)
    e = si.uniform_int8(11, name + ".e", (d.N, d.P, d.Q, d.K))
    desc = eoq.ConvDesc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, d.stride, d.pad)
    ud, wd, ed = dev(u), dev(w), dev(e)
    ws = torch.empty((max(max(eoq.Context.workspace_bytes(desc, op) for op in (0, 1, 2)), 16),), dtype=torch.uint8,
                     device="cuda")
    oshape = (d.N, d.P, d.Q, d.K)
    n_out = int(np.prod(oshape))
    # ---- forward with the fused epilogue, as the training step launches it
    sc = dev(np.array([119, -3, 5], dtype=np.int32))
    skip = si.uniform_int8(11, name + ".skip", oshape, 0, 127)
    y = torch.empty(oshape, dtype=torch.int8, device="cuda")
    un = torch.empty_like(y)
    mask = torch.empty(((n_out + 31) // 32,), dtype=torch.int32, device="cuda")
    skd = dev(skip)
    ep = ctx.epilogue(gamma=sc[0:1], b_post=sc[1:2], skip=skd, relu=1, b_next_pre=sc[2:3], y=y, u_next=un, mask=mask)
    ctx.conv_fwd(desc, ud, wd, ep=ep, ws=ws)
    yh, unh = y.cpu().numpy(), un.cpu().numpy()
    mh = np.unpackbits(mask.cpu().numpy().view(np.uint8), bitorder="little")[:n_out].reshape(oshape)
    for _ in range(200):
        n, p, q, k = (int(rng.integers(0, s)) for s in oshape)
        if _ < 40:                                   # include borders and the last tile
            n, p, q = d.N - 1, (0, d.P - 1)[_ % 2], (d.Q - 1, 0)[(_ // 2) % 2]
        t = int(oo.q_a1(np.array([fwd_sample(d, u, w, n, p, q, k)]))[0])
        z = oo.post_conv(np.array([t]), 119, -3, np.array([skip[n, p, q, k]]))
        yo, mo = oo.relu_q_a2(z)
        assert yh[n, p, q, k] == yo[0] and mh[n, p, q, k] == int(mo[0]), (name, n, p, q, k)
        assert unh[n, p, q, k] == oo.pre_bias(yo, 5)[0]
    assert yh.min() >= 0 and np.array_equal(unh, np.clip(yh.astype(np.int16) + 5, -127, 127))
    # ---- backward data: raw accumulators and the fused two-pass Q_e
    dacc = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.int32, device="cuda")
    sl = dev(np.array([0, 0, -15, 0], dtype=np.int32))
    ctx.conv_bwd_data(desc, ed, wd, dacc, sl[0:1], ws)
    e4 = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.int8, device="cuda")
    sums = torch.zeros((1,), dtype=torch.int64, device="cuda")
    ctx.conv_bwd_data_sq(desc, ed, wd, e4, sl[1:2], sl[2:3], -7, sl[3:4], sums, ws)
    M = int(dacc.abs().max().item())
    slh = sl.cpu().numpy()
    assert slh[0] == M and slh[1] == M
    r = oq.scale_exponent_int(M)
    assert slh[3] == -15 - 7 + r - 7
    dh, e4h = dacc.cpu().numpy(), e4.cpu().numpy()
    for _ in range(150):
        n, h, x, c = (int(rng.integers(0, s)) for s in dh.shape)
        if _ < 30:
            n, h, x = d.N - 1, (0, d.H - 1)[_ % 2], (d.W - 1, 0)[(_ // 2) % 2]
        want = dx_sample(d, e, w, n, h, x, c)
        assert dh[n, h, x, c] == want, (name, n, h, x, c)
        assert e4h[n, h, x, c] == int(np.clip(oq.rne_shift(np.array([want]), r - 7), -127, 127)[0])
    assert int(sums.item()) == int(e4h.astype(np.int64).sum())
    # the whole int8 tensor is the scale quantiser applied to the whole int32 tensor (checked on the device copy)
    codes, _ = oq.sq_int(dh[:2], 0) if int(np.abs(dh[:2]).max()) == M else (None, None)
    if codes is not None:
        assert np.array_equal(e4h[:2], codes)
    # ---- weight gradient
    g = torch.empty((d.K, d.R, d.S, d.C), dtype=torch.int32, device="cuda")
    gs = torch.zeros((1,), dtype=torch.int32, device="cuda")
    ctx.conv_bwd_weight(desc, ed, ud, g, gs, ws)
    gh = g.cpu().numpy()
    assert int(gs.item()) == int(np.abs(gh).max())
    for _ in range(60):
        k, r_, t_, c = (int(rng.integers(0, s)) for s in gh.shape)
        assert gh[k, r_, t_, c] == dw_sample(d, e, u, k, r_, t_, c), (name, k, r_, t_, c)
    # adjoint identity on the device results: <conv(u,W), e> = <W, dW(e,u)> = <u, dX(e,W)> (exact in int64)
    lhs_w = int((g.to(torch.int64) * wd.to(torch.int64)).sum().item())
    lhs_x = int((dacc.to(torch.int64) * ud.to(torch.int64)).sum().item())
    assert lhs_w == lhs_x
    assert ctx.status() == 0
    ctx.close()


@pytest.mark.parametrize("wl,batch", [("resnet18", 64), ("resnet50", 128)])
def test_full_batch_forward_equals_oracle_on_first_images(wl, batch):
    """No BatchNorm: the forward pass of an image does not depend on the rest of the batch, so the first two
    images of the full-size run must match an oracle run on those two images alone, bit for bit."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    x = si.batch_images(0, 0, batch, cfg["in_hw"])
    lab = si.batch_labels(0, 0, batch, cfg["classes"])
    g = FixupNet(cfg, batch, seed=0)
    loss = g.step(x, lab, 1, 8)
    o = OracleNet(cfg, 2, seed=0)
    yo, gap = o.forward(x[:2])
    # the GPU net has already updated its parameters; its forward activations were produced before that
    assert np.array_equal(g.y_out[:2].cpu().numpy(), yo)
    assert np.array_equal(g.gap[:2].cpu().numpy(), gap)
    assert np.array_equal(g.a0[:2].cpu().numpy(), o.trace["in.a"])
    assert np.isfinite(loss) and abs(loss - np.log(cfg["classes"])) < 1.0
    assert g.status() == 0
    # scale-quantiser invariant at any size: the largest code of every quantised gradient is 91..127 (or 0)
    for u in g.all_units:
        mc = g.slot_value(u.name + ".gmax")
        assert mc == 0 or 91 <= mc <= 127, (u.name, mc)
        assert int(u.w.abs().max().item()) <= 127


@pytest.mark.parametrize("wl,batch", [("resnet18", 64), ("resnet50", 128)])
def test_full_batch_inference_equals_oracle_on_sampled_images(wl, batch):
    """The int8 inference chain at the size and in the launch configuration the benchmark times (two half-batch
    chains, HIP graph replay): images sampled from both halves of the batch must match an oracle forward pass of
    those images alone (no BatchNorm: an image's forward pass does not depend on the rest of the batch)."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    x = si.batch_images(0, 0, batch, cfg["in_hw"])
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = FixupNet(cfg, batch, seed=0)
        g.x_in.copy_(torch.from_numpy(x).cuda())
        g.forward_inference()                            # eager once: one-time kernel attributes
        torch.cuda.synchronize()
        eager = g.gap.clone()
        g.gap.zero_(); g.y_out.zero_()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=stream):
            g.forward_inference()
        gr.replay()
        torch.cuda.synchronize()
    assert torch.equal(g.gap, eager)
    pick = [0, batch // 2 - 1, batch // 2, batch - 1]     # first and last image of each half-batch chain
    o = OracleNet(cfg, len(pick), seed=0)
    yo, gap = o.forward(x[pick])
    assert np.array_equal(g.y_out[pick].cpu().numpy(), yo)
    assert np.array_equal(g.gap[pick].cpu().numpy(), gap)
    assert g.status() == 0
