#!/usr/bin/env python3
"""Benchmark of the fused Distributed Lion step on one MI355X.

A "step" is one pass of the whole hot path -- worker momentum and sign for all
N workers, vote count, aggregation, weight update -- over one batch of
synthetic gradients that already sit in HBM.  Prints ONE JSON line with the
throughput in parameter-updates/s (d*N per step), the achieved fraction of the
HBM roofline for the fused kernel, and the CPU oracle timed on the host cores
on a bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, vendor figure


def algorithmic_bytes_per_step(d: int, N: int, g_bytes: int) -> int:
    """What the method must move per fused step: per update m in, m out, g in; per coordinate x in, x out."""
    return d * N * (4 + 4 + g_bytes) + 8 * d


def cpu_baseline(w, x, m, g, seconds_target: float = 12.0):
    """Time the CPU oracle (as it stands) on the first coordinates of the same workload."""
    import numpy as np
    import torch

    import oracle

    cores = min(len(os.sched_getaffinity(0)), 16)
    d_s = min(w.d, 16_000_000)
    xs = x[:d_s].cpu().numpy().copy()
    ms = m[:, :d_s].cpu().numpy().copy()
    gc = g[:, :d_s].cpu().contiguous()
    gs = gc.view(torch.int16).numpy().view(np.uint16).copy() if gc.dtype == torch.bfloat16 else gc.numpy().copy()
    oracle.step(xs.copy(), ms.copy(), gs, w.mode, w.beta1, w.beta2, w.lr, w.lam, threads=cores)   # warm
    t0 = time.perf_counter()
    oracle.step(xs.copy(), ms.copy(), gs, w.mode, w.beta1, w.beta2, w.lr, w.lam, threads=cores)
    one = max(time.perf_counter() - t0, 1e-6)
    reps = max(1, min(400, int(seconds_target / one)))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.step(xs, ms, gs, w.mode, w.beta1, w.beta2, w.lr, w.lam, threads=cores)
    dt = time.perf_counter() - t0
    return {
        "value": d_s * w.N * reps / dt,
        "unit": "param-updates/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"first {d_s} of {w.d} coordinates x {w.N} workers, {reps} steps, {cores} threads",
    }


def recorded_traffic(workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one.

    The counters cannot be read from inside this process; the figure is the one
    measured with ``rocprofv3 --pmc FETCH_SIZE`` / ``WRITE_SIZE`` over this very
    script and written into ``profiles/<kernel>_<workload>.md``.
    """
    import re

    import glob

    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"*_{workload}.md"))):
        try:
            with open(path) as f:
                m = re.search(r"traffic_bytes_per_launch:\s*(\d+)", f.read())
        except OSError:
            continue
        if m:
            return int(m.group(1))
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="gpt2s_avg8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of known size (1 GiB in, 1 GiB out, 5 times) so that "
                         "hardware counters collected over this run can be scaled against it")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py measures one GPU: every worker of the simulated run lives on the same device and "
              "no collectives are built; run it with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2404_00438_amd as dl
    from paper_2404_00438_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    dl.load_library()
    w = wl.CONFIGS[args.workload]
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    kernel = "dlion_step (fused"
    metric = "param-updates/s (d*N per fused step)"
    units = w.d * w.N                               # parameter-updates (or votes) per step
    bytes_per_launch = algorithmic_bytes_per_step(w.d, w.N, g_bytes)
    x = m = g = None
    # From 16 workers on the library runs the step as consecutive launches over 8 workers each when
    # it has somewhere to carry the votes: a workspace (flat buffers), else a counts array (tensor
    # lists), which then is an output of the step.
    ws_bytes = dl.dlion_step_workspace_bytes(w.d, w.N) if w.shapes is None else 0
    with_counts = w.N >= 16 and w.shapes is not None
    if w.g_dist == "packed_bernoulli":
        # vote-only pass: N pre-packed sign streams in, counts out
        W = dl.words_for(w.d)
        packed = wl.random_packed(w.N, W, dev, seed=w.seed)
        counts = torch.empty(w.d, dtype=torch.int16, device=dev)
        kernel = "dlion_aggregate (packed words in, uint16 counts out)"
        metric = "votes/s (d*N per vote-only pass)"
        bytes_per_launch = w.N * W * 8 + 2 * w.d

        def step():
            dl.dlion_aggregate(packed, w.d, counts)
    elif w.shapes is not None:
        numels = w.numels()
        xs = [wl.init_x(w, dev, tensor=k) for k in range(len(numels))]
        ms = [wl.init_m(w, dev, numel=n) for n in numels]
        gs = [wl.make_grads(w, 0, dev, tensor=k) for k in range(len(numels))]
        table = dl.SegTable(xs, ms, gs)
        counts = torch.empty(64 * table.total_words, dtype=torch.int16, device=dev) if with_counts else None
        kernel = f"dlion_step_mt (fused, {len(numels)} tensors"

        def step():
            dl.dlion_step_mt(table, w.N, w.mode, w.beta1, w.beta2, w.lr, w.lam, counts=counts)
    else:
        x = wl.init_x(w, dev)
        m = wl.init_m(w, dev)
        g = wl.make_grads(w, 0, dev)
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None

        def step():
            dl.dlion_step_ws(x, m, g, w.mode, w.beta1, w.beta2, w.lr, w.lam, workspace)
    if w.g_dist != "packed_bernoulli":
        if with_counts:
            kernel += ", counts output; launches over 8 workers each, 33.5 M coordinates at a time)"
            bytes_per_launch += 2 * w.d              # the counts the step hands back
        elif ws_bytes:
            kernel = kernel.replace("dlion_step ", "dlion_step_ws ")
            kernel += (f", no packed/counts output; launches over 8 workers each, 33.5 M coordinates at a time, "
                       f"votes carried in a {ws_bytes >> 20} MiB workspace)")
        else:
            kernel += ", no packed/counts output)"
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()                      # same stream the kernels are launched on (torch's current stream)
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = ev0.elapsed_time(ev1) / args.steps

    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9
    out = {
        "metric": metric,
        "value": units * args.steps / wall,
        "unit": metric.split(" ")[0],
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "d": w.d, "workers": w.N, "aggregation": "avg" if w.mode else "vote",
            "grad_dtype": str(w.g_dtype).replace("torch.", ""), "grad_dist": w.g_dist,
            "state_dtype": "float32", "kernel": kernel,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": recorded_traffic(w.name),
            "kernel_ms": kernel_ms,                  # all launches of one step
            "bytes_per_launch": bytes_per_launch,    # algorithmic bytes of one step
            "bytes_per_update": bytes_per_launch / units,
        },
    }
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "launches": 5}
    if not args.no_cpu_baseline and x is not None:
        out["cpu_baseline"] = cpu_baseline(w, x, m, g)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
