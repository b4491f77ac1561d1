"""Whole training steps at the sizes the metric is quoted on, on the path the benchmark runs (no tracing: fused
calls, two streams, half-batch forward chains, speculative backward-data calls), against the CPU oracle at the SAME
batch size: Fixup ResNet-50 at batch 128, ResNet-18 at batch 64, ResNet-20 at batch 128 (Section 5.1 workloads;
Eq.2-4, Eq.8-13 end to end).

Two steps per network, a fresh hashed batch each:
  step 0  launched eagerly at lr = 2^-8: every speculative call misses (no exponent known yet) and takes the
          exact path; the network stays alive;
  step 1  ONE REPLAY of the step captured into a HIP graph, at lr = 2^2 (2^1 for ResNet-18) written into the
          device-resident learning-rate slot: most speculative calls now hit, a few miss, and more than 1 % of the
          int8 weight codes move.  (One learning rate drives weights, scalars and the float classifier, and the
          rounding is deterministic: a rate that moves weight codes leaves the network dead after that step -- hence
          the small rate first.  A dead layer's all-zero error keeps a stale exponent, and the oracle refuses the
          resulting exponent gap by assertion.)
After each step: loss (1e-5 relative), every int8 weight tensor, every scalar code, every scalar gradient's code
and exponent, the float classifier and the device status word must equal the oracle's.

The oracle needs about 80 s per ResNet-50 step on 16 cores; progress lines keep the run from looking hung.
"""
import time

import numpy as np
import pytest

import seeded_inputs as si

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle.net import Net as OracleNet        # noqa: E402

CASES = [("resnet20", 128, [(1, 8), (1, -2)]),
         ("resnet18", 64, [(1, 8), (1, -1)]),
         ("resnet50", 128, [(1, 8), (1, -2)])]


def host(t):
    return t.detach().cpu().numpy()


def compare(g, o, tag):
    for u in g.all_units:
        assert np.array_equal(host(u.w), o.W[u.name]), (tag, u.name)
        if u.wt is not None:           # the transposed copy the next backward-data call multiplies with
            assert np.array_equal(host(u.wt).reshape(-1), o.W[u.name].transpose(3, 1, 2, 0).reshape(-1)), (tag, u.name, "wt")
    assert g.scalars() == {k: o.scal[k] for k in g.scalars()}, tag
    gc, ge = host(g.g_code), host(g.g_exp)
    for i, p in enumerate(g.sgrad_params):
        assert int(gc[i]) == o.trace[p + ".gs"] and int(ge[i]) == o.trace[p + ".Egs"], (tag, p)
    assert np.array_equal(host(g.Wfc), o.Wfc) and np.array_equal(host(g.bfc), o.bfc), tag
    # every exponent of the backward chain and of the weight gradients (the slots the kernels keep on the device)
    sl = host(g.slots32)
    n_exp = 0
    for u in g.all_units:
        for suffix, key in ((".E3", u.E3), (".E4", getattr(u, "E4", None)), (".Eg", u.name + ".Eg")):
            if key is not None and (u.name + suffix) in o.trace:
                assert int(sl[g.sl.names32[key]]) == o.trace[u.name + suffix], (tag, u.name + suffix)
                n_exp += 1
    for b in g.blocks:
        assert int(sl[g.sl.names32[b.name + ".E_in"]]) == o.trace[b.name + ".E_in"], (tag, b.name)
    assert n_exp > len(g.all_units)
    assert g.status() == 0, tag


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("wl,batch,sched", CASES, ids=[f"{c[0]}-b{c[1]}" for c in CASES])
def test_full_size_steps_eager_then_graph_replay(wl, batch, sched, capsys):
    from paper_2105_13890_amd.net import FixupNet
    cfg = si.WORKLOADS[wl]

    def say(msg):
        with capsys.disabled():
            print(f"[fullstep {wl} b{batch}] {msg}", flush=True)

    t0 = time.time()
    o = OracleNet(cfg, batch, seed=0)
    W0 = {k: v.copy() for k, v in o.W.items()}
    total = sum(v.size for v in W0.values())
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = FixupNet(cfg, batch, seed=0)
        graph = None
        for step, (m, j) in enumerate(sched):
            x = si.batch_images(0, step, batch, cfg["in_hw"])
            lab = si.batch_labels(0, step, batch, cfg["classes"])
            say(f"step {step}: oracle starts at {time.time() - t0:.0f} s")
            lo = o.step(x, lab, m, j)
            say(f"step {step}: oracle done at {time.time() - t0:.0f} s, loss {lo:.6f}")
            h0, m0 = g.spec_counters()
            if step == 0:
                lg = g.step(x, lab, m, j)                # eager (also sets one-time kernel attributes)
                graph = g.capture_step()                 # capturing runs nothing
            else:
                g.x_in.copy_(torch.from_numpy(x).cuda())
                g.labels.copy_(torch.from_numpy(lab).cuda())
                g.set_lr(m, j)
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                lg = float(g.loss.item())
            h1, m1 = g.spec_counters()
            assert lg == pytest.approx(lo, rel=1e-5), (step, lg, lo)
            compare(g, o, f"{wl} b{batch} step {step}")
            changed = sum(int((o.W[k] != W0[k]).sum()) for k in W0) / total
            say(f"step {step}: parity ok; weight codes changed vs init {changed:.5f}; "
                f"speculative calls hit {h1 - h0}, redone {m1 - m0}")
            if step == 0:
                assert h1 - h0 == 0 and m1 - m0 > 0      # nothing to speculate on yet
            else:
                assert h1 - h0 > 0, "the replay never took the one-evaluation path"
    assert changed > 0.01, "no weight code moved: the comparison of the update would be vacuous"
