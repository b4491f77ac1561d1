"""The optional stochastic-rounding update (beyond the paper; off by default): the library's _sr entry points and
whole training steps with it switched on, against the CPU oracle's implementation of the same counter-based hash --
bit for bit, like everything else.  Nothing here is a claim about the paper's own (deterministic) update rule."""
import zlib

import numpy as np
import pytest

import seeded_inputs as si

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle import ops as oo                   # noqa: E402
from oracle.net import Net as OracleNet        # noqa: E402


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def test_update_int8_sr_and_grad_update_sr():
    from paper_2105_13890_amd import eoq
    ctx = eoq.Context()
    seed, step, tid = 0xC0FFEE, 17, 0x12345678
    sr = dev(np.array([seed, step], dtype=np.int32))
    n = 16 * 3001 + 7
    W0 = si.uniform_int8(61, "w", (n,))
    g = si.uniform_int8(61, "g", (n,))
    for Eg, m, j in [(-17, 1, 0), (-12, 3, 2), (-9, 1, 0), (-7, 1, -3), (-40, 5, 0), (-75, 1, 0)]:
        w = dev(W0.copy())
        slots = dev(np.array([Eg, int(np.abs(g.astype(np.int64)).max()), m, j], dtype=np.int32))
        ctx.update_int8(w, dev(g), slots[0:1], slots[1:2], slots[2:4], sr_slot=sr, tensor_id=tid)
        want = oo.update_weights(W0, g, Eg, m, j, sr=(seed, tid, step))
        assert np.array_equal(host(w), want), (Eg, m, j)
        # the deterministic rule on the same inputs differs wherever a fraction of a code is at stake
        if Eg == -17:
            assert not np.array_equal(want, oo.update_weights(W0, g, Eg, m, j))
    # Q_g + Q_u + update + transposed copy in one pass
    K, R, S, Cc = 48, 3, 3, 32
    d = eoq.ConvDesc(1, 8, 8, Cc, K, R, S, 1, 1)
    acc = (si.uniform_int8(62, "acc", (K, R, S, Cc)).astype(np.int32) * 1117 + si.uniform_int8(62, "a2", (K, R, S, Cc)))
    Wk = si.uniform_int8(62, "wk", (K, R, S, Cc))
    for E3, m, j in [(-16, 1, 0), (-22, 7, 1), (-9, 1, 0)]:
        w, wt = dev(Wk.copy()), torch.zeros((Cc, R, S, K), dtype=torch.int8, device="cuda")
        sl = dev(np.array([int(np.abs(acc).max()), E3, m, j, 0, 0], dtype=np.int32))
        ctx.grad_update(d, dev(acc), sl[0:1], sl[1:2], -7, sl[2:4], w, wt=wt, exp_out=sl[4:5], max_code_out=sl[5:6],
                        sr_slot=sr, tensor_id=tid)
        gq, Egq = oo.sq_acc(acc, E3 - 7)
        want = oo.update_weights(Wk, gq, Egq, m, j, sr=(seed, tid, step))
        assert np.array_equal(host(w), want), (E3, m, j)
        assert np.array_equal(host(wt), want.transpose(3, 1, 2, 0))
        assert int(host(sl)[4]) == Egq
    # the step counter is advanced by a kernel
    ctx.sr_next_step(sr)
    assert host(sr).tolist() == [seed, step + 1]
    assert ctx.status() == 0
    ctx.close()


@pytest.mark.parametrize("wl,N,steps,lr,traced", [("tiny_basic", 4, 4, (1, 6), True), ("tiny_bottleneck", 3, 4, (3, 7), False),
                                                 ("resnet18", 2, 3, (1, 8), False)])
def test_network_steps_with_stochastic_rounding(wl, N, steps, lr, traced):
    """Whole steps at a learning rate where the deterministic rule moves (next to) no weight code: with stochastic
    rounding codes move in every step, and every parameter still equals the oracle's after every step."""
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]
    g, o = FixupNet(cfg, N, seed=0, trace=traced, sr_seed=1234), OracleNet(cfg, N, seed=0, sr_seed=1234)
    det = OracleNet(cfg, N, seed=0)
    moved_steps = 0
    for step in range(steps):
        x = si.batch_images(0, step, N, cfg["in_hw"])
        lab = si.batch_labels(0, step, N, cfg["classes"])
        before = {k: v.copy() for k, v in o.W.items()}
        lo, lg = o.step(x, lab, *lr), g.step(x, lab, *lr)
        assert lg == pytest.approx(lo, rel=1e-5)
        for u in g.all_units:
            assert np.array_equal(host(u.w), o.W[u.name]), (step, u.name)
        assert g.scalars() == {k: o.scal[k] for k in g.scalars()}, step
        assert g.status() == 0
        moved_steps += any((o.W[k] != before[k]).any() for k in before)
        if step == 0:
            det.step(x, lab, *lr)               # the paper's rule on the same step moves far fewer codes (none, mostly)
            moved_det = sum(int((det.W[k] != before[k]).sum()) for k in before)
            moved_sr = sum(int((o.W[k] != before[k]).sum()) for k in before)
            assert moved_sr > 4 * moved_det + 10, (moved_sr, moved_det)
    assert moved_steps == steps
    assert int(host(g.sr)[1]) == steps
