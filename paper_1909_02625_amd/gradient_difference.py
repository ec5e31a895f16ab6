"""Gradient-difference trace (Lemma 1; the quantity plotted in Section 5.4) on a synthetic workload.

    python -m paper_1909_02625_amd.gradient_difference [--workload resnet20] [--ticks 60] [--lr 0.01 0.001]

Runs DSP(p; m) with the library's gradient probe attached and prints, per learning rate, the relative
difference ||G^DSP_{x_k} - G^BP_{x_k}||_2 / ||G^BP_{x_k}||_2 of every block, averaged over windows of
mini-batches, and ||G^DSP - G^BP||_2 / (number of parameters of the block).  Inputs are seeded standard
normal images with uniform labels, one fresh mini-batch per tick (no dataset is read).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def trace(workload, dtype_name, ticks, lr, batch=None):
    import numpy as np
    import torch

    import paper_1909_02625_amd as D
    from paper_1909_02625_amd.marshal import build_gpu_blocks, destroy_blocks, round_like, to_dev
    from workloads import get_config, make_batch, make_params

    cfg = get_config(workload, batch=batch)
    dtype = D.DSP_BF16 if dtype_name == "bf16" else D.DSP_FP32
    K, p, m = cfg["K"], cfg["p"], cfg["m"]
    rng = np.random.default_rng(cfg["seed"])
    params = [make_params(layers, rng) for layers in cfg["blocks"]]
    blocks = build_gpu_blocks(cfg, params, dtype)
    probes = build_gpu_blocks(cfg, params, dtype, p=[0] * K, m=[0] * K)
    pl = D.dsp_pipeline_init(blocks, p, m, lr, cfg["beta"], cfg["wd"], ticks)
    pr = D.dsp_pipeline_init(probes, [0] * K, [0] * K, 0.0, 0.0, 0.0, ticks)
    D.dsp_pipeline_attach_gradient_probe(pl, pr)
    n_params = [int(D.dsp_block_query(b)["n_params"]) for b in blocks]
    rows = []
    try:
        for _ in range(ticks):
            x, y = make_batch(rng, cfg["input"], cfg["classes"])
            D.dsp_pipeline_step(pl, to_dev(round_like(x, dtype), dtype), torch.from_numpy(y).cuda())
            bid, diff, ref = D.dsp_pipeline_gradient_difference(pl, K)
            if bid >= 0:
                rows.append((bid, np.sqrt(diff), np.sqrt(ref)))
        losses = D.dsp_pipeline_losses(pl)
    finally:
        D.dsp_pipeline_destroy(pl)
        D.dsp_pipeline_destroy(pr)
        destroy_blocks(blocks)
        destroy_blocks(probes)
    return cfg, n_params, rows, losses


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet20")
    ap.add_argument("--dtype", default="fp32", choices=["fp32", "bf16"])
    ap.add_argument("--ticks", type=int, default=60)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--lr", type=float, nargs="+", default=[0.01, 0.001])
    ap.add_argument("--window", type=int, default=10)
    ap.add_argument("--json", action="store_true", help="one JSON line per learning rate instead of the table")
    a = ap.parse_args()
    import numpy as np

    for lr in a.lr:
        cfg, n_params, rows, losses = trace(a.workload, a.dtype, a.ticks, lr, a.batch)
        K = cfg["K"]
        rel = np.array([d / r for _, d, r in rows])
        per_param = np.array([d / np.asarray(n_params) for _, d, _ in rows])
        if a.json:
            print(json.dumps({"workload": a.workload, "dtype": a.dtype, "lr": lr, "p": list(cfg["p"]), "m": list(cfg["m"]),
                              "n_params": n_params, "batches": [int(b) for b, _, _ in rows],
                              "relative_difference": rel.tolist(), "difference_per_parameter": per_param.tolist()}))
            continue
        print("%s %s DSP(%s;%s) lr=%g  parameters per block %s" % (a.workload, a.dtype, ",".join(map(str, cfg["p"])),
                                                                    ",".join(map(str, cfg["m"])), lr, n_params))
        print("  mini-batches   " + "".join("  rel.diff block %d" % k for k in range(K)) +
              "".join("  per-param block %d" % k for k in range(K)))
        for w0 in range(0, len(rows), a.window):
            sl = slice(w0, min(w0 + a.window, len(rows)))
            print("  %4d .. %-4d   " % (rows[sl][0][0], rows[sl][-1][0]) +
                  "".join("  %16.4e" % v for v in rel[sl].mean(axis=0)) +
                  "".join("  %17.4e" % v for v in per_param[sl].mean(axis=0)))
        print("  loss: first %.4f last %.4f" % (losses[0], losses[-1]))


if __name__ == "__main__":
    main()
