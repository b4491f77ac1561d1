#!/usr/bin/env python3
"""Benchmark of the full-int8 Fixup-ResNet training step (forward + backward + int8 update) on one MI355X.

Prints ONE JSON line.  `value` is images/sec over the timed steps with the batches already resident in HBM: the timed
loop rotates over several distinct resident batches (one captured HIP graph per batch, each starting with the
device-side copy of its batch into the network's input buffer).  `roofline` is for the dominant kernel family (the
int8 MFMA implicit-GEMM convolution, forward launches), measured live with events on the stream the kernels run on.
`cpu_baseline` times the CPU oracle on a bounded sample (the same network at a small batch) on this machine's host
cores.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "resnet50_b128_step_hbm_traffic.txt")

# Learning rate m * 2^-j of the timed loop, per workload.  One rate drives weights, scalars and the float classifier,
# and the rounding is deterministic: a rate that moves int8 weight codes in every step (2^0 and above on these
# synthetic inputs) leaves the network dead (all-zero activations) within a few steps, and dead layers run faster
# than live ones.  The timed loop therefore uses the largest rate that keeps the network alive over its steps; the
# line reports what moved (weight codes, scalars), the pooled-feature mass at the end relative to the first step, and
# the speculative backward-data calls that hit / had to be redone per step, so that the reader sees what was timed.
# (scanned with --lr-j: 30 steps, scalars move, pooled-feature mass stays above 0.3, device flags 0)
LR = {"resnet20": (1, 4), "resnet18": (1, 6), "resnet34": (1, 6), "resnet50": (1, 6), "resnet110": (1, 5)}
DEFAULT_BATCH = {"resnet20": 128, "resnet18": 64, "resnet34": 64, "resnet50": 128, "resnet110": 128}
CPU_SAMPLE_BATCH = {"resnet20": 128, "resnet18": 32, "resnet34": 16, "resnet50": 16, "resnet110": 64}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def measured_fwd_traffic(workload: str, batch: int):
    """HBM bytes per forward-igemm launch from the committed rocprofv3 counter summary (ResNet-50 / batch 128 only)."""
    if workload != "resnet50" or batch != 128:
        return None
    try:
        m = re.search(r"fwd_igemm_hbm_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(TRAFFIC_PROFILE).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50", choices=sorted(LR))
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--batches", type=int, default=4, help="distinct resident batches the timed loop rotates over")
    ap.add_argument("--lr-j", type=int, default=None, help="learning rate 2^-j of the timed loop (default: per workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-layer", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--no-overlap", action="store_true", help="run the whole step on one stream")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every step from Python instead of replaying a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    import seeded_inputs as si
    from paper_2105_13890_amd.net import FixupNet

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    wl = args.workload
    cfg = si.WORKLOADS[wl]
    N = args.batch or DEFAULT_BATCH[wl]
    lr_m, lr_j = LR[wl]
    if args.lr_j is not None:
        lr_j = args.lr_j
    nb = max(1, args.batches)

    # Everything runs on one explicit stream (the library's side stream forks from it and joins it inside a step),
    # so that the step can be captured into a HIP graph: one graph launch per step instead of ~500 kernel launches
    # from Python.  The graph holds exactly the kernels of the eager step; --no-graph times the eager loop.
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    net = FixupNet(cfg, N, seed=0, overlap=not args.no_overlap)
    xs_host = [si.batch_images(0, b, N, cfg["in_hw"]) for b in range(nb)]
    ls_host = [si.batch_labels(0, b, N, cfg["classes"]) for b in range(nb)]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    ls = [torch.from_numpy(l).cuda() for l in ls_host]
    net.set_lr(lr_m, lr_j)
    W0 = [u.w.clone() for u in net.all_units]
    scal0 = net.scal.clone()
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.zero_()                         # writes 1 GiB
        torch.add(src, 1, out=dst)          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    def load_batch(b):                      # device-side copies, part of the timed region
        net.x_in.copy_(xs[b])
        net.labels.copy_(ls[b])

    load_batch(0)
    net.enqueue_step()                      # first step eager: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    gap0 = float(net.gap.abs().sum().item())
    if args.no_graph:
        def run_step(i):
            load_batch(i % nb)
            net.enqueue_step()
        launch = "eager"
    else:
        graphs = []
        for b in range(nb):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                load_batch(b)
                net.enqueue_step()
            graphs.append(g)

        def run_step(i):
            graphs[i % nb].replay()
        launch = f"hip graph replay (one graph per resident batch = batch copy + one step; {nb} batches in rotation)"
    for i in range(max(args.warmup - 1, 0)):
        run_step(1 + i)
    torch.cuda.synchronize()
    h0, m0 = net.spec_counters()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    h1, m1 = net.spec_counters()
    ms_per_step = dt / args.steps * 1e3
    img_s = N * args.steps / dt
    loss = float(net.loss.item())
    flags = net.status()
    gap1 = float(net.gap.abs().sum().item())
    tot_w = sum(w.numel() for w in W0)
    changed_w = sum(int((u.w != w0).sum().item()) for u, w0 in zip(net.all_units, W0)) / tot_w
    changed_s = int((net.scal != scal0).sum().item())

    # ---- one instrumented step: events around every convolution call, on ONE stream so that a call's duration is
    # its own (in the timed loop the weight-gradient chain overlaps the error chain on a second stream).  A queue
    # of plain elementwise kernels is enqueued first and keeps the stream busy while the host enqueues the step, so
    # that no event interval contains time the GPU spent waiting for the host. ----
    blk_a = torch.empty((1 << 29,), dtype=torch.uint8, device="cuda")
    blk_b = torch.empty_like(blk_a)
    net.prof = []
    overlap, net.overlap = net.overlap, False
    load_batch(0)
    for _ in range(60):
        torch.add(blk_a, 1, out=blk_b)
    net.enqueue_step()
    torch.cuda.synchronize()
    net.overlap = overlap
    prof_list, net.prof = net.prof, None
    del blk_a, blk_b

    # ---- forward passes alone, replayed as graphs: the training forward (masks and biased inputs kept for a backward
    # pass) and the inference chain (nothing kept: no masks, activations in two rotating buffers) ----
    fwd_only = infer = None
    if not args.no_graph:
        def time_graph(fn):
            fn()
            net._join()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                fn()
                net._join()
            g.replay()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / args.steps
        fdt = time_graph(net.forward)
        fwd_only = {"ms": round(fdt * 1e3, 4), "images_per_sec": round(N / fdt, 1),
                    "what": "training forward pass only (quantise input .. pooled features), graph replay, side outputs "
                            "for the backward pass kept"}
        if hasattr(net, "forward_inference"):
            idt = time_graph(net.forward_inference)
            infer = {"ms": round(idt * 1e3, 4), "images_per_sec": round(N / idt, 1),
                     "what": "int8 inference chain (quantise input .. pooled features): no masks, no stored "
                             "activations, graph replay"}

    # algorithmic bytes of the forward convolutions: int8 input + int8 filters read, int8 outputs (y and / or the
    # next layer's biased input), 1-bit mask, shortcut read, wide Q_a1 output where it is kept
    fwd_bytes = 0.0
    layer_bytes = {}
    for u in net.all_units:
        d = u.desc
        n_out = d.N * d.P * d.Q * d.K
        b = d.N * d.H * d.W * d.C + d.K * d.R * d.S * d.C
        # wide shortcut conv output (2 or 4 bytes per element, as allocated) | mask + one int8 out
        b += u.t.element_size() * n_out if not u.relu else n_out / 8 + n_out
        layer_bytes[u.name] = b
    for b in net.blocks:
        last = b.units[-1].desc
        n_out = last.N * last.P * last.Q * last.K
        extra = b.ds.t.element_size() * n_out if b.ds else n_out           # shortcut read
        if getattr(b, "y_written", True):
            extra += n_out                                                  # block outputs written twice (y, u_next)
        layer_bytes[b.units[-1].name] += extra
    fwd_bytes = sum(layer_bytes.values())
    agg = {}
    rows = []
    for kind, unit, work, e0, e1 in prof_list:
        ms = e0.elapsed_time(e1)
        a = agg.setdefault(kind, [0.0, 0.0, 0])
        a[0] += work
        a[1] += ms
        a[2] += 1
        rows.append((kind, unit, work, ms))
    # streaming passes (requantisation, update, input quantisation): algorithmic bytes over event-timed duration
    hbm = {k[4:]: {"calls": v[2], "ms": round(v[1], 4), "gbs": round(v[0] / (v[1] * 1e-3) / 1e9, 1),
                   "frac_of_hbm_peak": round(v[0] / (v[1] * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
           for k, v in agg.items() if k.startswith("hbm_")}
    agg = {k: v for k, v in agg.items() if not k.startswith("hbm_")}
    conv = {k: {"calls": v[2], "ms": round(v[1], 4), "tops": round(v[0] / (v[1] * 1e-3) / 1e12, 2)}
            for k, v in agg.items()}
    tot_ops = sum(v[0] for v in agg.values())
    tot_ms = sum(v[1] for v in agg.values())
    fwd = agg["conv_fwd"]
    fwd_tops = fwd[0] / (fwd[1] * 1e-3) / 1e12
    if args.per_layer:
        # every convolution call against min(MFMA peak, arithmetic intensity x HBM peak); forward rows use the
        # layer's algorithmic bytes, the backward kinds the bytes their operands and outputs take at stored width
        units = {u.name: u for u in net.all_units}
        print(f"{'kind':18s} {'layer':10s} {'GOP':>8s} {'MB':>8s} {'us':>8s} {'TOP/s':>8s} {'GB/s':>8s} {'bound TOP/s':>11s} {'of bound':>8s}",
              file=sys.stderr)
        for kind, unit, work, ms in rows:
            if kind.startswith("hbm_"):
                print(f"{kind:18s} {unit:10s} {'':8s} {work / 1e6:8.1f} {ms * 1e3:8.1f} {'':8s} {work / (ms * 1e-3) / 1e9:8.0f} "
                      f"{'(HBM 8000)':>11s} {work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS:8.2f}", file=sys.stderr)
                continue
            d = units[unit].desc
            n_in, n_out, n_w = d.N * d.H * d.W * d.C, d.N * d.P * d.Q * d.K, d.K * d.R * d.S * d.C
            if kind == "conv_fwd":
                byts = layer_bytes[unit]
            elif kind == "conv_bwd_weight":
                byts = n_in + n_out + 4 * n_w
            elif kind == "conv_bwd_data":
                byts = n_out + n_w + n_in + n_in / 8
            else:
                byts = n_in + n_w + n_out
            bound = min(PEAK_INT8_TOPS, work / byts * PEAK_HBM_GBS / 1e3)
            tops = work / (ms * 1e-3) / 1e12
            print(f"{kind:18s} {unit:10s} {work / 1e9:8.2f} {byts / 1e6:8.1f} {ms * 1e3:8.1f} {tops:8.1f} "
                  f"{byts / (ms * 1e-3) / 1e9:8.0f} {bound:11.0f} {tops / bound:8.2f}", file=sys.stderr)

    steps_done = args.steps
    out = {
        "metric": "int8 training images/sec (fwd+bwd+update); conv int8 TOPS as % of MFMA peak",
        "value": round(img_s, 2),
        "unit": "images/sec",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"Fixup {wl} full-int8 training step, batch {N}, {cfg['in_hw']}x{cfg['in_hw']}x3 "
                               f"~N(0,1) inputs, {cfg['classes']} classes, lr={lr_m}*2^{-lr_j}", "global_batch": N,
                   "resident_batches": nb, "launch": launch,
                   "streams": 1 if args.no_overlap else 2,
                   "stream_use": "one stream" if args.no_overlap else
                                 "forward of the blocks: two half-batch chains; backward: error chain | weight-gradient chain"},
        "loss": loss,
        "device_flags": flags,
        "timed_loop": {"speculative_calls_per_step": round((h1 - h0 + m1 - m0) / steps_done, 2),
                       "spec_hits_per_step": round((h1 - h0) / steps_done, 2),
                       "spec_misses_per_step": round((m1 - m0) / steps_done, 2),
                       "weight_codes_changed_vs_init": round(changed_w, 6),
                       "scalar_codes_changed_vs_init": changed_s, "scalar_codes": int(net.scal.numel()) - 1,
                       "pooled_feature_mass_vs_first_step": round(gap1 / gap0, 4) if gap0 else None,
                       "note": "a hit codes the backward-data sums in one evaluation, a miss is redone through the 16-bit "
                               "intermediate (same result); a dead network (feature mass near 0) would run faster than a live one"},
        "conv_tops_all": round(tot_ops / (tot_ms * 1e-3) / 1e12, 2),
        "conv_pct_of_int8_peak": round(100.0 * tot_ops / (tot_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
        "conv_ms_single_stream_sum": round(tot_ms, 3),
        "conv": conv,
        "hbm_passes": hbm,
        "forward_only": fwd_only,
        "inference": infer,
        "roofline": {"bound": "mfma", "kernel": "igemm_kernel (forward convolution launches of one step)",
                     "achieved": round(fwd_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": round(fwd_tops / PEAK_INT8_TOPS, 4),
                     "traffic": measured_fwd_traffic(wl, N),
                     "launches": fwd[2], "avg_launch_us": round(fwd[1] * 1e3 / fwd[2], 2),
                     "algorithmic_ops_per_launch": round(fwd[0] / fwd[2]),
                     "algorithmic_bytes_per_launch": round(fwd_bytes / fwd[2]),
                     "hbm_gbs_at_algorithmic_bytes": round(fwd_bytes / (fwd[1] * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak_at_algorithmic_bytes": round(fwd_bytes / (fwd[1] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "note": "int8 multiply-add counted as 2 ops; algorithmic ops 2*N*P*Q*K*C*R*S summed over the forward "
                             "launches of one step divided by their summed event-timed durations, taken in one extra step "
                             "launched on ONE stream with whole-batch launches behind a queue of filler kernels (so that no "
                             "interval contains host launch time; the timed steps run the same kernel on half batches in two "
                             "concurrent chains, where a launch's duration is not its own); traffic = measured HBM bytes per "
                             "launch, read from the committed rocprofv3 counter summary under profiles/ (FETCH_SIZE + "
                             "WRITE_SIZE, scaled by a 1 GiB copy); the forward pass as a whole moves its algorithmic bytes at "
                             "the HBM fraction given, i.e. it sits between the two roofs; measured MFMA ceilings on this chip: "
                             "4.9 POP/s with all-zero operands, 3.3 POP/s with random int8 operands (power-limited)"},
    }

    if not args.no_cpu_baseline:
        from oracle.net import Net as OracleNet
        nbc = min(CPU_SAMPLE_BATCH[wl], N)
        onet = OracleNet(cfg, nbc, seed=0)
        t0 = time.perf_counter()
        onet.step(xs_host[0][:nbc], ls_host[0][:nbc], lr_m, lr_j)
        cdt = time.perf_counter() - t0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": round(nbc / cdt, 4), "unit": "images/sec", "cores": cores, "kind": "oracle",
                               "cpu": cpu_model(),
                               "sample": f"one full training step of the same network on the first {nbc} images "
                                         f"of the batch ({cdt:.1f} s); the oracle's convolutions are per-image loops, so a "
                                         f"full batch of {N} takes {N / nbc:.0f}x as long ({cdt * N / nbc:.0f} s extrapolated)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
