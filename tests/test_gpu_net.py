"""GPU parity of whole training steps: every tensor the HIP path produces (activations, masks,
errors, gradients, exponents, updated parameters) against the CPU oracle, bit for bit; loss to 1e-5."""
import numpy as np
import pytest

import seeded_inputs as si

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle.net import Net as OracleNet        # noqa: E402


def host(t):
    return t.detach().cpu().numpy()


def compare_traces(gnet, onet, tag=""):
    """Every name both sides recorded must agree exactly."""
    T, G = onet.trace, gnet.trace
    n_cmp = 0
    sl = host(G["slots32"])
    for name, want in T.items():
        if isinstance(want, np.ndarray):
            if name not in G:
                continue
            got = host(G[name])
            if name.endswith(".mask"):
                got = np.unpackbits(got.view(np.uint8), bitorder="little")[:want.size].astype(bool).reshape(want.shape)
            if name in ("head.logits", "head.d"):
                assert np.array_equal(got, want), (tag, name)
            else:
                assert got.shape == want.shape, (tag, name, got.shape, want.shape)
                assert np.array_equal(got.astype(np.int64), want.astype(np.int64)), (tag, name)
            n_cmp += 1
        elif name.endswith((".E3", ".E4", ".Eg", ".E_in")) or name in ("head.E", "pool.E"):
            key = name
            if name.endswith(".E3"):
                unit = name[:-3]
                key = next(u for u in gnet.all_units if u.name == unit).E3
            assert int(sl[gnet.sl.names32[key]]) == want, (tag, name)
            n_cmp += 1
    # scalar gradients
    gc, ge = host(G["g_code"]), host(G["g_exp"])
    for i, p in enumerate(gnet.sgrad_params):
        assert int(gc[i]) == T[p + ".gs"] and int(ge[i]) == T[p + ".Egs"], (tag, p)
    return n_cmp


def compare_params(gnet, onet, tag=""):
    for u in gnet.all_units:
        assert np.array_equal(host(u.w), onet.W[u.name]), (tag, u.name)
    assert gnet.scalars() == {k: onet.scal[k] for k in gnet.scalars()}, tag
    if gnet.classes:
        assert np.array_equal(host(gnet.Wfc), onet.Wfc), tag
        assert np.array_equal(host(gnet.bfc), onet.bfc), tag


def changed_fraction(before, after):
    ch = sum(int((after[k] != before[k]).sum()) for k in before)
    return ch / sum(v.size for v in before.values())


def test_lone_block_config(request):
    """One Fixup basic block 16->16 on 8x32x32x16: one full fwd + bwd + int8 update, seed 0."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS["block16"]
    N = 8
    a = si.uniform_int8(0, "block.a", (N, 32, 32, 16))
    e0 = si.uniform_int8(0, "block.e0", (N, 32, 32, 16))
    g, o = FixupNet(cfg, N, seed=0, trace=True), OracleNet(cfg, N, seed=0)
    compare_params(g, o, "init")
    W0 = {k: v.copy() for k, v in o.W.items()}
    for step, (m, j) in enumerate([(1, 10), (3, 9)]):
        yo, eo, Eo = o.block_step(a, e0, -7, m, j)
        yg, eg = g.block_step(a, e0, -7, m, j)
        assert np.array_equal(host(yg), yo)
        assert np.array_equal(host(eg), eo) and g.slot_value("s0b0.E_in") == Eo
        assert compare_traces(g, o, f"step{step}") > 10
        compare_params(g, o, f"step{step}")
        assert g.status() == 0
    assert changed_fraction(W0, o.W) > 0.01


@pytest.mark.parametrize("wl,N,steps,lr", [("tiny_basic", 4, 3, (1, 1)), ("tiny_bottleneck", 3, 3, (3, 2)),
                                           ("resnet20", 128, 2, (1, -2)),
                                           # the ImageNet-shaped nets at a batch the oracle finishes in seconds
                                           ("resnet18", 2, 2, (1, 2)), ("resnet50", 2, 1, (1, 0))])
def test_network_steps(wl, N, steps, lr):
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    g, o = FixupNet(cfg, N, seed=0, trace=True), OracleNet(cfg, N, seed=0)
    compare_params(g, o, "init")
    W0 = {k: v.copy() for k, v in o.W.items()}
    for step in range(steps):
        x = si.batch_images(0, step, N, cfg["in_hw"])
        lab = si.batch_labels(0, step, N, cfg["classes"])
        lo = o.step(x, lab, *lr)
        lg = g.step(x, lab, *lr)
        assert lg == pytest.approx(lo, rel=1e-5)
        assert compare_traces(g, o, f"{wl} step{step}") > 20
        compare_params(g, o, f"{wl} step{step}")
        assert g.status() == 0
    assert changed_fraction(W0, o.W) > 0.01, "test would be vacuous: no weight code moved"


@pytest.mark.parametrize("wl,N,steps,lr", [("tiny_basic", 4, 3, (1, 1)), ("tiny_bottleneck", 4, 3, (3, 2)),
                                           ("tiny_bottleneck", 3, 2, (3, 2)),     # odd batch: whole-batch forward
                                           ("resnet50", 2, 1, (1, 0)), ("resnet50", 4, 1, (1, 0)),
                                           # the paper's other two networks
                                           ("resnet34", 2, 1, (1, 2)), ("resnet110", 4, 2, (1, -2))])
def test_network_steps_untraced(wl, N, steps, lr):
    """The same comparison on the path the benchmark runs: without tracing the step uses its fused calls (ReLU
    backward and Q_e(e1*gamma) inside the merge pass, Q_g + update + transpose in one kernel, pool backward with the
    stem's mask, two half-batch forward chains, deferred updates on the side stream).  Loss and every parameter
    after every step must equal the oracle's."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    g, o = FixupNet(cfg, N, seed=0), OracleNet(cfg, N, seed=0)
    W0 = {k: v.copy() for k, v in o.W.items()}
    for step in range(steps):
        x = si.batch_images(0, step, N, cfg["in_hw"])
        lab = si.batch_labels(0, step, N, cfg["classes"])
        lo = o.step(x, lab, *lr)
        lg = g.step(x, lab, *lr)
        assert lg == pytest.approx(lo, rel=1e-5)
        compare_params(g, o, f"{wl} step{step}")
        # scalar gradients as well (their sums come from the fused kernels)
        gc, ge = host(g.g_code), host(g.g_exp)
        for i, p in enumerate(g.sgrad_params):
            assert int(gc[i]) == o.trace[p + ".gs"] and int(ge[i]) == o.trace[p + ".Egs"], (wl, step, p)
        assert g.status() == 0
    assert changed_fraction(W0, o.W) > 0.01, "test would be vacuous: no weight code moved"


@pytest.mark.parametrize("wl,N", [("tiny_basic", 4), ("tiny_bottleneck", 3), ("resnet20", 8), ("resnet18", 2),
                                  ("resnet50", 4)])
def test_forward_inference_equals_oracle(wl, N):
    """The int8 inference chain (forward only, every training side output switched off) gives the oracle's forward
    pass bit for bit, writes no ReLU mask and leaves the stored per-layer inputs of a training step alone."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    g, o = FixupNet(cfg, N, seed=0), OracleNet(cfg, N, seed=0)
    # scalars off their initial values (the same on both sides), so that every bias and multiplier matters
    sc = host(g.scal).copy()
    for i, name in enumerate(g.scal_names):
        sc[i] += (i % 7) - 3
        o.scal[name] = int(sc[i])
    g.scal.copy_(torch.from_numpy(sc).cuda())
    x = si.batch_images(0, 5, N, cfg["in_hw"])
    yo, gap = o.forward(x)
    g.x_in.copy_(torch.from_numpy(x).cuda())
    for u in g.all_units:                       # sentinels: a training side output that gets written would show
        if u.mask is not None:
            u.mask.fill_(0x5a5a5a5a)
        if u.relu and u is not g.stem:
            u.u.fill_(77)
    g.forward_inference()
    torch.cuda.synchronize()
    assert np.array_equal(host(g.y_out), yo)
    assert np.array_equal(host(g.gap), gap)
    for u in g.all_units:
        if u.mask is not None:
            assert bool((u.mask == 0x5a5a5a5a).all()), u.name
        if u.relu and u is not g.stem:
            assert bool((u.u == 77).all()), u.name
    assert g.status() == 0
    # and a training step afterwards is unaffected by the buffers the inference pass borrowed
    lab = si.batch_labels(0, 5, N, cfg["classes"])
    lo, lg = o.step(x, lab, 1, 3), g.step(x, lab, 1, 3)
    assert lg == pytest.approx(lo, rel=1e-5)
    compare_params(g, o, f"{wl} step after inference")
