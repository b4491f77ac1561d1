#!/usr/bin/env python3
"""Learning-rate scan for the small-batch trajectory test, on the CPU oracle alone.

Runs Fixup ResNet-18 at batch 1 for a number of consecutive training steps (a fresh hashed batch per step)
at several learning rates lr = m * 2^-j and records, per rate: in how many steps at least one int8 weight code
moved, the fraction of weight codes that differ from the initial ones at the end, how many scalar codes moved,
the largest scalar magnitude (biases that run away switch layers off), the pooled-feature sum at the end (0 =
the network is dead) and whether the oracle's own range assertions held.  Nothing here touches the GPU path.

    python tests/golden/scan_trajectory_lr.py [--steps 200] [--batch 1] > tests/golden/trajectory_lr_scan.txt
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import seeded_inputs as si                  # noqa: E402
from oracle.net import Net                  # noqa: E402

RATES = [(1, 4), (3, 5), (1, 3), (5, 5), (1, 2)]


def scan(batch, steps, rates):
    cfg = si.WORKLOADS["resnet18"]
    print(f"# oracle-only scan: resnet18, batch {batch}, {steps} steps, fresh hashed batch per step, seed 0")
    print("# lr  steps_with_weight_movement  weight_codes_changed_vs_init  scalars_moved/of  max|scalar|  "
          "last_gap_abs_sum  ok")
    for m, j in rates:
        o = Net(cfg, batch, seed=0)
        W0 = {k: v.copy() for k, v in o.W.items()}
        total = sum(v.size for v in W0.values())
        prev = {k: v.copy() for k, v in W0.items()}
        moving, ok, done = 0, "yes", 0
        try:
            for step in range(steps):
                x = si.batch_images(0, step, batch, cfg["in_hw"])
                lab = si.batch_labels(0, step, batch, cfg["classes"])
                o.step(x, lab, m, j)
                moved = sum(int((o.W[k] != prev[k]).sum()) for k in prev)
                prev = {k: v.copy() for k, v in o.W.items()}
                moving += moved > 0
                done = step + 1
        except AssertionError as e:                       # exponent gap or scalar range: the run diverged
            ok = f"assertion at step {done}: {e}"
        changed = sum(int((o.W[k] != W0[k]).sum()) for k in W0) / total
        sc_moved = sum(1 for k, v in o.scal.items() if v != (128 if k.endswith(".g") else 0))
        gap = int(np.abs(o.trace["gap.sum"]).sum()) if "gap.sum" in o.trace else -1
        print(f"{m}*2^-{j}  {moving}/{done}  {changed:.6f}  {sc_moved}/{len(o.scal)}  "
              f"{max(abs(v) for v in o.scal.values())}  {gap}  {ok}", flush=True)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--batch", type=int, default=1)
    a = ap.parse_args()
    scan(a.batch, a.steps, RATES)
