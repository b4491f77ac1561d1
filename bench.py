#!/usr/bin/env python3
"""Benchmark of the full-int8 Fixup-ResNet training step (forward + backward + int8 update) on one MI355X.

Prints ONE JSON line.  `value` is images/sec over the timed steps with the batch already resident in
HBM.  `roofline` is for the dominant kernel family (the int8 MFMA implicit-GEMM convolution, forward
launches), measured live with events on the stream the kernels run on.  `cpu_baseline` times the CPU
oracle on a bounded sample (the same network at a small batch) on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published
# HBM bytes per forward-igemm launch of the ResNet-50 / batch-128 step, from two rocprofv3 --pmc runs (FETCH_SIZE,
# WRITE_SIZE) scaled by a 1 GiB elementwise kernel: profiles/resnet50_b128_step_hbm_traffic.txt
MEASURED_FWD_TRAFFIC_BYTES = {"resnet50": 93.7e6}

# learning rate m * 2^-j per workload.  With one learning rate for weights and scalars and deterministic
# rounding, a rate large enough to move >= 1% of the int8 weight codes per step drives the biases far enough
# in a few steps on a repeated batch to switch whole layers off; the timed loop therefore uses a small rate
# that keeps the network alive (kernel work per step does not depend on the values either way).
LR = {"resnet20": (1, 4), "resnet18": (1, 8), "resnet34": (1, 8), "resnet50": (1, 8), "resnet110": (1, 4)}
DEFAULT_BATCH = {"resnet20": 128, "resnet18": 64, "resnet34": 64, "resnet50": 128, "resnet110": 128}
CPU_SAMPLE_BATCH = {"resnet20": 128, "resnet18": 32, "resnet34": 16, "resnet50": 16, "resnet110": 64}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50", choices=sorted(LR))
    ap.add_argument("--batch", type=int, default=0)
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

    # Everything runs on one explicit stream (the library's side stream forks from it and joins it inside a step),
    # so that the step can be captured into a HIP graph: one graph launch per step instead of ~700 kernel launches
    # from Python.  The graph holds exactly the kernels of the eager step; --no-graph times the eager loop.
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    net = FixupNet(cfg, N, seed=0, overlap=not args.no_overlap)
    x = si.batch_images(0, 0, N, cfg["in_hw"])
    lab = si.batch_labels(0, 0, N, cfg["classes"])
    net.x_in.copy_(torch.from_numpy(x).cuda())
    net.labels.copy_(torch.from_numpy(lab).cuda())
    net.set_lr(lr_m, lr_j)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.zero_()                         # writes 1 GiB
        torch.add(src, 1, out=dst)          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    net.enqueue_step()                      # first step eager: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph = None if args.no_graph else net.capture_step()
    run_step = net.enqueue_step if graph is None else graph.replay
    for _ in range(max(args.warmup - 1, 0)):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    img_s = N * args.steps / dt
    loss = float(net.loss.item())
    flags = net.status()

    # ---- one instrumented step: events around every convolution call, on ONE stream so that a call's duration is
    # its own (in the timed loop the weight-gradient chain overlaps the error chain on a second stream) ----
    net.prof = []
    overlap, net.overlap = net.overlap, False
    net.enqueue_step()
    torch.cuda.synchronize()
    net.overlap = overlap
    prof_list, net.prof = net.prof, None
    # ---- forward pass alone (input quantisation -> pooled integer features; the int8 inference chain of the same
    # kernels, still writing the masks and biased inputs a backward pass would need), replayed as a graph ----
    fwd_only = None
    if graph is not None:
        net.forward()
        net._join()
        torch.cuda.synchronize()
        gf = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gf, stream=stream):
            net.forward()
            net._join()
        gf.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            gf.replay()
        torch.cuda.synchronize()
        fdt = (time.perf_counter() - t0) / args.steps
        fwd_only = {"ms": round(fdt * 1e3, 4), "images_per_sec": round(N / fdt, 1),
                    "what": "forward pass only (quantise input .. pooled features), graph replay, training side outputs kept"}

    # algorithmic bytes of the forward convolutions: int8 input + int8 filters read, int8 outputs (y and / or the
    # next layer's biased input), 1-bit mask, shortcut read, wide Q_a1 output where it is kept
    fwd_bytes = 0.0
    for u in net.all_units:
        d = u.desc
        n_out = d.N * d.P * d.Q * d.K
        fwd_bytes += d.N * d.H * d.W * d.C + d.K * d.R * d.S * d.C
        # wide shortcut conv output (2 or 4 bytes per element, as allocated) | mask + one int8 out
        fwd_bytes += u.t.element_size() * n_out if not u.relu else n_out / 8 + n_out
    for b in net.blocks:
        last = b.units[-1].desc
        n_out = last.N * last.P * last.Q * last.K
        fwd_bytes += n_out                                                      # block outputs are written twice (y, u_next)
        fwd_bytes += b.ds.t.element_size() * n_out if b.ds else n_out           # shortcut read
    agg = {}
    rows = []
    for kind, unit, work, e0, e1 in prof_list:
        ms = e0.elapsed_time(e1)
        a = agg.setdefault(kind, [0.0, 0.0, 0])
        a[0] += work
        a[1] += ms
        a[2] += 1
        rows.append((kind, unit, work, ms))
    net.prof = None
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
        for kind, unit, work, ms in rows:
            if kind.startswith("hbm_"):
                print(f"{kind:16s} {unit:10s} {work / 1e6:10.2f} MB  {ms:8.4f} ms {work / (ms * 1e-3) / 1e9:8.1f} GB/s",
                      file=sys.stderr)
            else:
                print(f"{kind:16s} {unit:10s} {work / 1e9:10.2f} GOP {ms:8.4f} ms {work / (ms * 1e-3) / 1e12:8.1f} TOP/s",
                      file=sys.stderr)

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
                   "launch": "eager" if graph is None else "hip graph replay (one graph = one step)",
                   "streams": 1 if args.no_overlap else 2,
                   "stream_use": "one stream" if args.no_overlap else
                                 "forward of the blocks: two half-batch chains; backward: error chain | weight-gradient chain"},
        "loss": loss,
        "device_flags": flags,
        "conv_tops_all": round(tot_ops / (tot_ms * 1e-3) / 1e12, 2),
        "conv_pct_of_int8_peak": round(100.0 * tot_ops / (tot_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
        "conv_ms_of_step": round(tot_ms, 3),
        "conv": conv,
        "hbm_passes": hbm,
        "forward_only": fwd_only,
        "roofline": {"bound": "mfma", "kernel": "igemm_kernel (forward convolution launches of one step)",
                     "achieved": round(fwd_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                     "frac": round(fwd_tops / PEAK_INT8_TOPS, 4),
                     "traffic": MEASURED_FWD_TRAFFIC_BYTES.get(wl) if N == DEFAULT_BATCH[wl] else None,
                     "launches": fwd[2], "avg_launch_us": round(fwd[1] * 1e3 / fwd[2], 2),
                     "algorithmic_ops_per_launch": round(fwd[0] / fwd[2]),
                     "algorithmic_bytes_per_launch": round(fwd_bytes / fwd[2]),
                     "hbm_gbs_at_algorithmic_bytes": round(fwd_bytes / (fwd[1] * 1e-3) / 1e9, 1),
                     "note": "int8 multiply-add counted as 2 ops; algorithmic ops 2*N*P*Q*K*C*R*S summed over the forward "
                             "launches of one step divided by their summed event-timed durations, taken in one extra step "
                             "launched eagerly on ONE stream with whole-batch launches (the timed steps run the same kernel "
                             "on half batches in two concurrent chains, where a launch's duration is not its own); traffic = measured HBM "
                             "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy); measured MFMA "
                             "ceilings on this chip: 4.9 POP/s with all-zero operands, 3.3 POP/s with random int8 operands "
                             "(power-limited)"},
    }

    if not args.no_cpu_baseline:
        from oracle.net import Net as OracleNet
        nb = min(CPU_SAMPLE_BATCH[wl], N)
        onet = OracleNet(cfg, nb, seed=0)
        xs, ls = x[:nb], lab[:nb]
        t0 = time.perf_counter()
        onet.step(xs, ls, lr_m, lr_j)
        cdt = time.perf_counter() - t0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": round(nb / cdt, 4), "unit": "images/sec", "cores": cores, "kind": "oracle",
                               "sample": f"one full training step of the same network on the first {nb} images "
                                         f"of the batch ({cdt:.1f} s)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
