#!/usr/bin/env python3
"""Benchmark of the DSP block step on one MI355X.

A "step" is one pipeline tick: every block of DSP(p; m) runs forward(a), recompute+backward(b) and
its momentum-SGD update on its own HIP stream, on synthetic inputs that are already resident in
HBM.  The default workload is the largest configuration that fits one GPU: the ResNet-18-shaped
ImageNet-sized net in bf16, K = 4 blocks, batch 256.  Prints ONE JSON line (the fields are described
in the README).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet20|resnet56|resnet18|resnet50_conv4x|vgg19|resnet164|resnet1001|tiny2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2500.0}  # MI355X dense MFMA
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet18")
    ap.add_argument("--dtype", default=None, choices=[None, "fp32", "bf16"])
    ap.add_argument("--batch", type=int, default=None, help="override the mini-batch size (not the headline number)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the CPU-oracle baseline leg (0 = skip)")
    ap.add_argument("--profile-steps", type=int, default=5)
    ap.add_argument("--kernels", type=int, default=12, help="how many kernels (heaviest first) the JSON line lists")
    ap.add_argument("--straggler", type=int, nargs=2, metavar=("BLOCK", "MICROSECONDS"), default=None,
                    help="straggler emulation: block BLOCK's stream idles this long before its work in every tick "
                         "(not the headline number)")
    ap.add_argument("--schedule", default=None, metavar="P;M",
                    help='another DSP(p; m) for the workload\'s K blocks, e.g. "2,2,0;6,3,0" (not the headline number)')
    ap.add_argument("--spare", type=int, default=0,
                    help="spare entries in every queue between two blocks: lets neighbouring blocks drift apart by more "
                         "than one tick (results are unchanged)")
    ap.add_argument("--random-stragglers", type=float, nargs="+", metavar="PERCENT", default=None,
                    help="after the timed ticks, one more series of --steps ticks per value: in every tick each block "
                         "independently, with probability 1/3, first idles PERCENT %% of the undisturbed tick time "
                         "(robustness experiment of Section 6); reported next to the headline number")
    ap.add_argument("--straggler-seed", type=int, default=0)
    return ap.parse_args()


class Workload:
    """Library objects + resident synthetic inputs for one configuration."""

    def __init__(self, name, dtype_name, batch, max_ticks, schedule=None, spare=0):
        import numpy as np
        import torch

        import paper_1909_02625_amd as D
        from paper_1909_02625_amd.marshal import block_shapes, build_gpu_blocks, round_like, to_dev
        from workloads import get_config, make_batch, make_params
        from workloads.gen import make_error_gradient

        self.D, self.torch = D, torch
        self.cfg = cfg = get_config(name, batch=batch)
        if schedule is not None:
            ps, ms = schedule.split(";")
            cfg["p"], cfg["m"] = tuple(int(v) for v in ps.split(",")), tuple(int(v) for v in ms.split(","))
            if len(cfg["p"]) != cfg["K"] or len(cfg["m"]) != cfg["K"]:
                sys.exit("bench.py: --schedule needs %d values of p and of m" % cfg["K"])
        self.dtype_name = dtype_name or cfg["dtypes"][0]
        self.dtype = D.DSP_BF16 if self.dtype_name == "bf16" else D.DSP_FP32
        rng = np.random.default_rng(cfg["seed"])
        self.params = [make_params(layers, rng) for layers in cfg["blocks"]]
        self.blocks = build_gpu_blocks(cfg, self.params, self.dtype, spare=spare)
        self.shapes = block_shapes(cfg)
        self.N = cfg["input"][0]
        self.external = cfg.get("classes") is None
        nbuf = 4
        self.batches = []
        for _ in range(nbuf):
            x, y = make_batch(rng, cfg["input"], cfg["classes"])
            g = None
            if self.external:
                g = to_dev(round_like(make_error_gradient(rng, self.shapes[-1], cfg.get("grad_std", 0.1)), self.dtype),
                           self.dtype)
            self.batches.append((to_dev(x, self.dtype), None if y is None else torch.from_numpy(y).cuda(), g))
        self.pl = None
        self.tick = 0
        self.fill = max(sum(cfg["p"][:k]) + cfg["m"][k] for k in range(cfg["K"]))
        if not self.external:
            self.pl = D.dsp_pipeline_init(self.blocks, cfg["p"], cfg["m"], cfg["lr"], cfg["beta"], cfg["wd"], max_ticks)
        else:
            self.out = torch.empty(int(np.prod(self.shapes[-1])), device="cuda",
                                   dtype=torch.bfloat16 if self.dtype == D.DSP_BF16 else torch.float32)
            self.gin = torch.empty(int(np.prod(self.shapes[0])), device="cuda", dtype=self.out.dtype)
        torch.cuda.synchronize()

    def step(self):
        D, cfg = self.D, self.cfg
        x, y, g = self.batches[self.tick % len(self.batches)]
        if self.pl is not None:
            D.dsp_pipeline_step(self.pl, x, y)
        else:  # a lone mid-network block fed with an external error gradient
            b, m = self.blocks[0], cfg["m"][0]
            if self.tick - m >= 0:
                D.dsp_block_step(b, self.tick, x, self.out, None, None, self.tick - m, g, self.gin)
                D.dsp_param_update(b, cfg["lr"], cfg["beta"], cfg["wd"])
            else:
                D.dsp_block_forward(b, self.tick, x, self.out)
        self.tick += 1

    def sync(self):
        if self.pl is not None:
            self.D.dsp_pipeline_sync(self.pl)
        self.torch.cuda.synchronize()

    def close(self):
        from paper_1909_02625_amd.marshal import destroy_blocks
        if self.pl is not None:
            self.D.dsp_pipeline_destroy(self.pl)
        destroy_blocks(self.blocks)


def cpu_baseline(name, batch, seconds):
    """The CPU oracle (as is) on a bounded sample of the same workload: images/s of one steady-state tick.

    Small workloads: the oracle's own pipeline on the first ticks at the full mini-batch, timed over the steady
    ticks.  Workloads whose tick would take the oracle minutes (ImageNet-sized): every block once through
    forward(a) + recompute/backward(b) + update -- exactly the work of one steady tick -- on its real layer
    shapes at a reduced mini-batch that fits the time budget; the sample string says which."""
    import numpy as np

    from oracle import dsp_oracle as O
    from workloads import count_macs, get_config, make_batch, make_params
    from workloads.gen import make_error_gradient

    cfg = get_config(name, batch=batch)
    N = cfg["input"][0]
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    shapes = [tuple(cfg["input"])]
    from workloads.configs import block_output_shape
    for layers in cfg["blocks"]:
        shapes.append(tuple(block_output_shape(layers, shapes[-1])))
    gmac_img = sum(count_macs(layers, shapes[k]) for k, layers in enumerate(cfg["blocks"])) * 4 / 1e9
    est_tick_s = gmac_img * N / (2.0 * cores)  # ~2 GMAC/s per core for the plain loops
    if est_tick_s <= seconds / 6:
        rng = np.random.default_rng(cfg["seed"])
        params = [make_params(layers, rng) for layers in cfg["blocks"]]
        orc = O.build_cnn_oracle(cfg, params)
        fill = max(sum(cfg["p"][:k]) + cfg["m"][k] for k in range(cfg["K"]))
        ext = cfg.get("classes") is None
        steady, t_steady, t_start, tick = 0, 0.0, time.perf_counter(), 0
        while True:
            x, y = make_batch(rng, cfg["input"], cfg["classes"])
            t0 = time.perf_counter()
            orc.tick(x, y, top_gradient=(lambda a, out: make_error_gradient(rng, out.shape, 0.1).astype(np.float64)) if ext else None)
            dt = time.perf_counter() - t0
            if tick >= fill:
                steady += 1
                t_steady += dt
            tick += 1
            if steady >= 1 and time.perf_counter() - t_start > seconds:
                break
            if steady >= 8:
                break
        return {"value": N * steady / t_steady, "unit": "images/s", "cores": cores, "kind": "oracle",
                "sample": "%d steady ticks (after %d fill ticks) of %s at batch %d, fp64, plain C loops + OpenMP over the batch"
                          % (steady, fill, name, N)}
    # one steady tick's work, block by block, at a reduced mini-batch
    nb = N
    while nb > 4 and gmac_img * nb / (2.0 * cores) > seconds / 2:
        nb //= 2
    cfg = get_config(name, batch=nb)
    rng = np.random.default_rng(cfg["seed"])
    params = [make_params(layers, rng) for layers in cfg["blocks"]]
    orc = O.build_cnn_oracle(cfg, params)
    shapes = [(nb,) + s[1:] for s in shapes]
    ext = cfg.get("classes") is None
    t_tick = 0.0
    for k, blk in enumerate(orc.blocks):
        h = rng.standard_normal(shapes[k])
        g = rng.standard_normal(shapes[k + 1]) * 0.1
        t0 = time.perf_counter()
        out, _ = blk.forward(h)                                   # forward(a)
        if k == cfg["K"] - 1 and not ext:
            _, g = orc.loss.value_and_grad(out, rng.integers(0, cfg["classes"], nb))
        _, gx = blk.vjp(h, g)                                      # recompute(b) + backward(b)
        blk.set_param_list(orc.opt[k].step(blk.param_list(), gx))  # update
        t_tick += time.perf_counter() - t0
    return {"value": nb / t_tick, "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": "one steady tick's work of %s (each of the %d blocks once: forward + recompute/backward + update on its "
                      "real layer shapes) at batch %d instead of %d, %.1f s, fp64, plain C loops + OpenMP over the batch"
                      % (name, cfg["K"], nb, N, t_tick)}


def hbm_traffic(workload, dtype_name, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload, or None.

    The summary holds one line "TRAFFIC <kernel> <fetch bytes> <write bytes>" per kernel: FETCH_SIZE and
    WRITE_SIZE per dispatch, each scaled by what the same counter reads for a copy kernel of known size.
    """
    path = os.path.join(ROOT, "profiles", "rocprofv3_pmc_hbm_traffic_%s_%s_pipeline_tick.txt" % (workload, dtype_name))
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] == "TRAFFIC" and f[1] == kernel:
            return float(f[2]) + float(f[3])
    return None


def calibration_copy(torch):
    """A plain copy of known size (64 MiB read, 64 MiB written), outside the timed region: the reference
    that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters when this script runs under --pmc."""
    src = torch.ones(16 << 20, device="cuda", dtype=torch.float32)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the K blocks share it on K HIP streams); --gpus %d is not supported"
              % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_1909_02625_amd as D
    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    calibration_copy(torch)
    total_ticks = a.warmup + 16 + a.steps * (1 + len(a.random_stragglers or [])) + a.profile_steps + 4
    w = Workload(a.workload, a.dtype, a.batch, total_ticks, a.schedule, a.spare)
    if a.straggler is not None:
        if w.pl is None:
            sys.exit("bench.py: --straggler needs a pipeline of several blocks")
        w.D.dsp_pipeline_set_delay(w.pl, a.straggler[0], a.straggler[1])
    # untimed: at least the ticks that fill the pipeline plus two steady ones (the first steady tick of a block
    # allocates its second buffer set), whatever --warmup says
    warm = max(a.warmup, w.fill + 2)
    for _ in range(warm):
        w.step()
    w.sync()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        w.step()
    w.sync()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / a.steps
    value = w.N * a.steps / (t1 - t0)

    # per-kernel time of the same ticks, from event pairs recorded around every launch on its own stream
    table = []
    if a.profile_steps > 0:
        # the same ticks once more with the K chains on ONE stream, so that no two kernels overlap and every
        # launch's duration (event pair around it) is that kernel's own; the markers dsp_profile_start / _stop
        # launch let a rocprofv3 kernel trace of this command be cut to exactly these launches
        if w.pl is not None:
            D.dsp_pipeline_set_single_stream(w.pl, True)
        D.dsp_profile_start(400000)
        for _ in range(a.profile_steps):
            w.step()
        w.sync()
        table = D.dsp_profile_stop()
        if w.pl is not None:
            D.dsp_pipeline_set_single_stream(w.pl, False)
    roof, kernels, conv_util = None, [], None
    if table:
        tot_ms = sum(k["ms"] for k in table)
        peak = PEAK_TFLOPS[w.dtype_name]
        for k in sorted(table, key=lambda k: -k["ms"]):
            avg_us = 1e3 * k["ms"] / k["launches"]
            rate = k["units"] / (k["ms"] * 1e-3) if k["ms"] > 0 else 0.0
            kernels.append({"name": k["name"], "launches_per_step": k["launches"] / a.profile_steps,
                            "avg_us": round(avg_us, 2), "share": round(k["ms"] / tot_ms, 4),
                            ("tflops" if k["unit_kind"] == "flop" else "gbs"):
                                round(rate / (1e12 if k["unit_kind"] == "flop" else 1e9), 2)})
        conv = [k for k in table if k["unit_kind"] == "flop"]
        if conv:
            conv_util = 100.0 * sum(k["units"] for k in conv) / (sum(k["ms"] for k in conv) * 1e-3) / (peak * 1e12)
        dom = max(table, key=lambda k: k["ms"])
        if dom["unit_kind"] == "flop":
            ach = dom["units"] / (dom["ms"] * 1e-3) / 1e12
            roof = {"bound": "mfma", "kernel": dom["name"], "achieved": round(ach, 3), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(ach / peak, 4), "traffic": hbm_traffic(a.workload, w.dtype_name, dom["name"]),
                    "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
                    "flop_per_launch": dom["units"] / dom["launches"]}
        else:
            ach = dom["units"] / (dom["ms"] * 1e-3) / 1e9
            roof = {"bound": "hbm", "kernel": dom["name"], "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": hbm_traffic(a.workload, w.dtype_name, dom["name"]),
                    "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
                    "bytes_per_launch": dom["units"] / dom["launches"]}
    # Section 6 (robustness): the same ticks with blocks that are late at random
    stragglers = None
    if a.random_stragglers:
        import numpy as np
        if w.pl is None:
            sys.exit("bench.py: --random-stragglers needs a pipeline of several blocks")
        stragglers = []
        for pct in a.random_stragglers:
            srng = np.random.default_rng(a.straggler_seed)
            delay_us = int(round(ms * 1e3 * pct / 100.0))
            hits = 0
            w.sync()
            ts = time.perf_counter()
            for _ in range(a.steps):
                for k in range(w.cfg["K"]):
                    late = srng.random() < 1.0 / 3.0
                    hits += int(late)
                    D.dsp_pipeline_set_delay(w.pl, k, delay_us if late else 0)
                w.step()
            w.sync()
            te = time.perf_counter()
            ms_s = (te - ts) * 1e3 / a.steps
            stragglers.append({"block_slow_down_pct": pct, "delay_us": delay_us, "probability": "1/3 per block and tick",
                               "delayed_block_ticks": hits, "ms_per_step": round(ms_s, 4),
                               "slow_down_pct": round(100.0 * (ms_s / ms - 1.0), 2)})
        for k in range(w.cfg["K"]):
            D.dsp_pipeline_set_delay(w.pl, k, 0)
    w.close()

    base = None
    if a.cpu_seconds > 0:
        base = cpu_baseline(a.workload, a.batch, a.cpu_seconds)

    cfg = w.cfg
    out = {
        "metric": "images/sec per DSP block step (fwd+recompute+bwd+update); conv MFMA util %",
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": warm,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype_name == "fp32" else "bf16", "data": "synthetic",
        "config": {"workload": "%s: DSP(%s;%s), K=%d blocks on %d HIP streams, batch %d x %dx%dx%d, one pipeline tick per step"
                               % (a.workload, ",".join(map(str, cfg["p"])), ",".join(map(str, cfg["m"])), cfg["K"],
                                  cfg["K"], cfg["input"][0], cfg["input"][1], cfg["input"][2], cfg["input"][3]),
                   "lr": cfg["lr"], "momentum": cfg["beta"],
                   **({"straggler": {"block": a.straggler[0], "microseconds": a.straggler[1]}} if a.straggler else {}),
                   **({"spare_queue_entries": a.spare} if a.spare else {})},
        **({"random_stragglers": stragglers} if stragglers else {}),
        "conv_mfma_util_pct": None if conv_util is None else round(conv_util, 3),
        # sum of all kernel durations of a tick (over the K streams); K * ms_per_step minus this is stream idle time
        "kernel_time_ms_per_step": None if not table else round(sum(k["ms"] for k in table) / a.profile_steps, 4),
        "library_build_id": D.dsp_build_id(), "roofline": roof, "cpu_baseline": base, "kernels": kernels[:a.kernels],
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
