#!/usr/bin/env python3
"""Writes tests/golden/trajectory_<config>_<dtype>[_b<batch>_hw<hw>].txt: the CPU oracle's free-running DSP loss
trajectory on one seeded synthetic workload, next to the trajectories of two perturbed runs of the SAME oracle.

Imports only oracle/ and workloads/.  The GPU parity tests replay the same seeded mini-batches through the
library and compare its losses with the stored ones, so a trajectory that takes the oracle minutes is computed
once, here.  The two perturbed runs measure how far apart two correct evaluations of the same recursion drift:
  run B: every stored tensor additionally rounded the way the compared arithmetic type keeps it
         (fp32 comparisons: storage="fp32" against plain fp64; bf16 comparisons: initial parameters moved by one
         fp32 ulp, storage="bf16" in both);
  run C: initial parameters moved by one fp32 ulp (another random sign pattern), otherwise identical to run A.
Columns: tick, mini-batch of the loss (-1 while the pipeline fills), loss of run A, |B - A| / |A|, |C - A| / |A|.

    python tests/golden/make_trajectory_spread.py --config resnet20 --dtype fp32 [--ticks 50] [--batch N] [--hw S]
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import dsp_oracle as O  # noqa: E402
from workloads import get_config, make_batch, make_params  # noqa: E402
from workloads.gen import perturb_one_ulp as one_ulp  # noqa: E402


def run(cfg, params, storage, ticks, bf16_inputs):
    rng = np.random.default_rng(cfg["seed"])
    for layers in cfg["blocks"]:
        make_params(layers, rng)  # advance the stream exactly as the tests do before drawing mini-batches
    orc = O.build_cnn_oracle(cfg, params, storage=storage)
    losses, batches = [], []
    for _ in range(ticks):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        if bf16_inputs:
            x = O.round_bf16(x)
        rec = orc.tick(x, y)
        losses.append(rec["loss"] if rec["loss"] is not None else float("nan"))
        batches.append(rec["loss_batch"] if rec["loss_batch"] is not None else -1)
    return np.array(losses), batches


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", required=True)
    ap.add_argument("--dtype", required=True, choices=["fp32", "bf16"])
    ap.add_argument("--ticks", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--hw", type=int, default=None)
    ap.add_argument("--out-dir", default=os.path.dirname(os.path.abspath(__file__)))
    a = ap.parse_args()
    cfg = get_config(a.config, batch=a.batch, hw=a.hw)
    ticks = a.ticks or cfg["steps"]
    rng = np.random.default_rng(cfg["seed"])
    params = [make_params(layers, rng) for layers in cfg["blocks"]]
    bf16 = a.dtype == "bf16"
    t0 = time.time()
    A, batches = run(cfg, params, "bf16" if bf16 else None, ticks, bf16)
    print("run A %.0f s" % (time.time() - t0), flush=True)
    if bf16:
        B, _ = run(cfg, one_ulp(params, 101), "bf16", ticks, True)
    else:
        B, _ = run(cfg, params, "fp32", ticks, False)
    print("run B %.0f s" % (time.time() - t0), flush=True)
    C, _ = run(cfg, one_ulp(params, 202), "bf16" if bf16 else None, ticks, bf16)
    print("run C %.0f s" % (time.time() - t0), flush=True)
    name = "trajectory_%s_%s" % (a.config, a.dtype)
    if a.batch is not None or a.hw is not None:
        name += "_b%d_hw%d" % (cfg["input"][0], cfg["input"][2])
    path = os.path.join(a.out_dir, name + ".txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_trajectory_spread.py --config %s --dtype %s --ticks %d%s%s\n"
                % (a.config, a.dtype, ticks, "" if a.batch is None else " --batch %d" % a.batch,
                   "" if a.hw is None else " --hw %d" % a.hw))
        f.write("# workload: %s, input %s, DSP(%s;%s), lr %g, momentum %g, seed %d; oracle storage mode of run A: %s\n"
                % (a.config, "x".join(map(str, cfg["input"])), ",".join(map(str, cfg["p"])), ",".join(map(str, cfg["m"])),
                   cfg["lr"], cfg["beta"], cfg["seed"], "bf16" if bf16 else "none (fp64)"))
        f.write("# tick batch loss_A gap_B gap_C\n")
        for t in range(ticks):
            if batches[t] < 0:
                f.write("%d -1 nan nan nan\n" % t)
            else:
                f.write("%d %d %.17g %.3e %.3e\n" % (t, batches[t], A[t], abs(B[t] - A[t]) / abs(A[t]), abs(C[t] - A[t]) / abs(A[t])))
    print("wrote", path)


if __name__ == "__main__":
    main()
