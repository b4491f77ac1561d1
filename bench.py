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

    net = FixupNet(cfg, N, seed=0)
    x = si.batch_images(0, 0, N, cfg["in_hw"])
    lab = si.batch_labels(0, 0, N, cfg["classes"])
    net.x_in.copy_(torch.from_numpy(x).cuda())
    net.labels.copy_(torch.from_numpy(lab).cuda())
    net.set_lr(lr_m, lr_j)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        net.enqueue_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        net.enqueue_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    img_s = N * args.steps / dt
    loss = float(net.loss.item())
    flags = net.status()

    # ---- one instrumented step: events around every convolution call ----
    net.prof = []
    net.enqueue_step()
    torch.cuda.synchronize()
    agg = {}
    rows = []
    for kind, unit, work, e0, e1 in net.prof:
        ms = e0.elapsed_time(e1)
        a = agg.setdefault(kind, [0.0, 0.0, 0])
        a[0] += work
        a[1] += ms
        a[2] += 1
        rows.append((kind, unit, work, ms))
    net.prof = None
    conv = {k: {"calls": v[2], "ms": round(v[1], 4), "tops": round(v[0] / (v[1] * 1e-3) / 1e12, 2)}
            for k, v in agg.items()}
    tot_ops = sum(v[0] for v in agg.values())
    tot_ms = sum(v[1] for v in agg.values())
    fwd = agg["conv_fwd"]
    fwd_tops = fwd[0] / (fwd[1] * 1e-3) / 1e12
    if args.per_layer:
        for kind, unit, work, ms in rows:
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
                               f"~N(0,1) inputs, {cfg['classes']} classes, lr={lr_m}*2^{-lr_j}", "global_batch": N},
        "loss": loss,
        "device_flags": flags,
        "conv_tops_all": round(tot_ops / (tot_ms * 1e-3) / 1e12, 2),
        "conv_pct_of_int8_peak": round(100.0 * tot_ops / (tot_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
        "conv_ms_of_step": round(tot_ms, 3),
        "conv": conv,
        "roofline": {"bound": "mfma", "kernel": "igemm_kernel (forward convolution launches of one step)",
                     "achieved": round(fwd_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                     "frac": round(fwd_tops / PEAK_INT8_TOPS, 4), "traffic": None,
                     "note": "int8 multiply-add counted as 2 ops; algorithmic ops 2*N*P*Q*K*C*R*S summed over the "
                             "launches divided by their summed durations"},
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
