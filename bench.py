#!/usr/bin/env python3
"""Benchmark of the fused Distributed Lion step on one MI355X.

A "step" is one pass of the whole hot path -- worker momentum and sign for all
N workers, vote count, aggregation, weight update -- over one batch of
synthetic gradients that already sit in HBM.  Prints ONE JSON line: the
throughput in parameter-updates/s (d*N per step) of the headline workload (the
largest one that stands for a training run of the paper: d = 350 M, 32 workers),
the achieved fraction of the HBM roofline of its kernel, plain memory-rate
ceilings measured in the same run, the CPU oracle timed on the host cores on a
bounded sample of the same workload, and (unless --headline-only) a short
measurement of every other workload so that each one's roofline fraction is on
record.
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
HEADLINE = "gpt350m_vote32"
# A process that allocates tens of GB soon after another large process has exited runs 4 % slower for its
# whole life (measured: started at once after a 67 GB process 18.5 ms per step, started 3 s or more later
# 17.8 ms, and 17.8 ms for 600 steps on end; after a 250 GB process 4 s are not enough, 8 s are).  The
# device reports all of its memory as free at once, so the wait cannot be replaced by a check.  Every
# measuring process therefore waits before it allocates: this long when it does not know what ran before
# it, SETTLE_CHILD_S in the processes this script starts itself (their predecessor held 70 GB at most).
SETTLE_S = 12.0
SETTLE_CHILD_S = 4.0


def algorithmic_bytes_per_step(d: int, N: int, g_bytes: int) -> int:
    """What the method must move per fused step: per update m in, m out, g in; per coordinate x in, x out."""
    return d * N * (4 + 4 + g_bytes) + 8 * d


def oracle_inputs(w, x, m, g, d_s):
    import numpy as np
    import torch

    xs = x[:d_s].cpu().numpy().copy()
    ms = m[:, :d_s].cpu().numpy().copy()
    gc = g[:, :d_s].cpu().contiguous()
    gs = gc.view(torch.int16).numpy().view(np.uint16).copy() if gc.dtype == torch.bfloat16 else gc.numpy().copy()
    return xs, ms, gs


def time_oracle(w, xs, ms, gs, threads, seconds_target):
    import oracle

    args = (w.mode, w.beta1, w.beta2, w.lr, w.lam)
    oracle.step(xs.copy(), ms.copy(), gs, *args, threads=threads)   # warm
    t0 = time.perf_counter()
    oracle.step(xs.copy(), ms.copy(), gs, *args, threads=threads)
    one = max(time.perf_counter() - t0, 1e-6)
    reps = max(1, min(400, int(seconds_target / one)))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.step(xs, ms, gs, *args, threads=threads)
    return reps, time.perf_counter() - t0


def cpu_baseline(w, x, m, g):
    """The CPU oracle (as it stands) on the first coordinates of the same workload: all host threads
    this process may use (at most 16, the box's share per GPU), and one thread on a smaller sample."""
    avail = len(os.sched_getaffinity(0))
    cores = min(avail, 16)
    d_all = min(w.d, max(1 << 20, 128_000_000 // w.N))
    d_one = max(1 << 18, d_all // 8)
    xs, ms, gs = oracle_inputs(w, x, m, g, d_all)
    reps, dt = time_oracle(w, xs, ms, gs, cores, 12.0)
    reps1, dt1 = time_oracle(w, xs[:d_one].copy(), ms[:, :d_one].copy(), gs[:, :d_one].copy(), 1, 6.0)
    return {
        "value": d_all * w.N * reps / dt,
        "unit": "param-updates/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"first {d_all} of {w.d} coordinates x {w.N} workers, {reps} steps, {cores} threads",
        "single_thread": {
            "value": d_one * w.N * reps1 / dt1,
            "unit": "param-updates/s",
            "cores": 1,
            "sample": f"first {d_one} of {w.d} coordinates x {w.N} workers, {reps1} steps, 1 thread",
        },
        "nproc": os.cpu_count(),
        "usable_cpus": avail,
    }


def recorded_traffic(workload: str, entry: str = "step"):
    """HBM bytes per step from the committed rocprofv3 --pmc summary of this workload, if there is one.

    The counters cannot be read from inside this process; the figure is the one
    measured with ``rocprofv3 --pmc FETCH_SIZE`` / ``WRITE_SIZE`` over this very
    script and written into ``profiles/<kernel>_<workload>.md``.  Returns
    (bytes or None, path relative to the repository or None).
    """
    import glob
    import re

    prefix = "dlion_aggregate" if workload == "packed256_1b" and entry == "step" else f"dlion_{entry}"
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"{prefix}_{workload}.md"))):
        try:
            with open(path) as f:
                m = re.search(r"traffic_bytes_per_launch:\s*(\d+)", f.read())
        except OSError:
            continue
        if m:
            return int(m.group(1)), os.path.relpath(path, ROOT)
    return None, None


def timed(step, steps, warmup):
    """(kernel ms per step from HIP events on the launch stream, wall seconds for all steps)"""
    import torch

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()                      # same stream the kernels are launched on (torch's current stream)
    for _ in range(steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return ev0.elapsed_time(ev1) / steps, wall


def memory_ceilings(dev):
    """Plain memory-rate probes of the library (no arithmetic of the method), best over a few caps on the
    resident waves and numbers of loads in flight per wave: a copy, a read (8 rows per wave, nothing
    written), and 16 rows read per row written (the byte mix of counting 256 packed streams into uint16
    counts)."""
    import torch

    import paper_2404_00438_amd as dl

    n = 1 << 29                                        # 2 GiB of fp32 per row
    src = torch.empty((16, n // 8), dtype=torch.float32, device=dev).normal_()
    flat = src.view(-1)
    dst = torch.empty(n, dtype=torch.float32, device=dev)
    out = {}
    for key, (s, d, rows, write) in {
        "copy_ceiling_gbs": (flat[:n], dst, 1, True),
        "read_ceiling_gbs": (src[:8], dst[: n // 8], 8, False),
        "mix16to1_ceiling_gbs": (src, dst[: n // 8], 16, True),
    }.items():
        best = 0.0
        for in_flight in sorted({min(rows, 2), min(rows, 4), rows}):
            for cap in (0, 8, 16, 24):
                def probe():
                    return dl.dlion_membench(s, d, rows=rows, write=write, loads_in_flight=in_flight,
                                             waves_per_cu=cap)
                rd, wr = probe()
                ms, _ = timed(probe, 6, 2)
                best = max(best, (rd + wr) / (ms * 1e-3) / 1e9)
        out[key] = best
    del src, dst, flat
    torch.cuda.empty_cache()
    return out


ENTRIES = ("step", "worker_step", "aggregate", "apply", "aggregate_apply", "aggregate_encode", "apply_encoded")


def run_workload(name, steps, warmup, dev, with_cpu_baseline=False, entry="step"):
    """Measure one workload; returns the record for the JSON line.  entry != "step": one of the unfused
    calls on the same state instead of the fused step (flat workloads with gradients only)."""
    import torch

    import paper_2404_00438_amd as dl
    from paper_2404_00438_amd import workloads as wl

    w = wl.CONFIGS[name]
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    kernel = "dlion_step (fused, no packed/counts output"
    metric = "param-updates/s (d*N per fused step)"
    units = w.d * w.N                               # parameter-updates (or votes) per step
    bytes_per_step = algorithmic_bytes_per_step(w.d, w.N, g_bytes)
    x = m = g = None
    if w.g_dist == "packed_bernoulli":
        # vote-only pass: N pre-packed sign streams in, counts out
        W = dl.words_for(w.d)
        packed = wl.random_packed(w.N, W, dev, seed=w.seed, row_stride=wl.padded_words(W))
        counts = torch.empty(w.d, dtype=torch.int16, device=dev)
        kernel = "dlion_aggregate (packed words in, uint16 counts out)"
        metric = "votes/s (d*N per vote-only pass)"
        bytes_per_step = w.N * W * 8 + 2 * w.d

        def step():
            dl.dlion_aggregate(packed, w.d, counts)
    elif w.shapes is not None:
        numels = w.numels()
        xs = [wl.init_x(w, dev, tensor=k) for k in range(len(numels))]
        ms = [wl.init_m(w, dev, numel=n) for n in numels]
        gs = [wl.make_grads(w, 0, dev, tensor=k) for k in range(len(numels))]
        table = dl.SegTable(xs, ms, gs)
        ws_bytes = dl.dlion_step_mt_workspace_bytes(table.total_tiles, w.N)
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
        kernel = f"dlion_step_mt_ws (fused, {len(numels)} tensors, no packed/counts output"

        def step():
            dl.dlion_step_mt(table, w.N, w.mode, w.beta1, w.beta2, w.lr, w.lam, workspace=workspace)
    else:
        # rows padded so that every worker's row starts on a 1 KB boundary (the layout the header recommends)
        stride = wl.padded_stride(w.d)
        x = wl.init_x(w, dev)
        m = wl.init_m(w, dev, row_stride=stride)
        g = wl.make_grads(w, 0, dev, row_stride=stride)
        ws_bytes = dl.dlion_step_workspace_bytes(w.d, w.N)
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
        kernel = "dlion_step_ws (fused, no packed/counts output" if ws_bytes else kernel

        def step():
            dl.dlion_step_ws(x, m, g, w.mode, w.beta1, w.beta2, w.lr, w.lam, workspace)

        if entry != "step":
            # the unfused calls, on packed words / counts / planes that the library's own calls produced
            W = dl.words_for(w.d)
            packed = torch.zeros((w.N, wl.padded_words(W)), dtype=torch.int64, device=dev)[:, :W]
            counts = torch.empty(w.d, dtype=torch.int16, device=dev)
            planes = dl.dlion_delta_planes(w.N, w.mode)
            delta = torch.zeros((planes, wl.padded_words(W)), dtype=torch.int64, device=dev)[:, :W]
            dl.dlion_worker_step(m, g, packed, w.beta1, w.beta2)
            dl.dlion_aggregate(packed, w.d, counts)
            dl.dlion_aggregate_encode(packed, w.d, w.mode, delta)
            calls = {
                "worker_step": (lambda: dl.dlion_worker_step(m, g, packed, w.beta1, w.beta2),
                                w.d * w.N * (8 + g_bytes) + w.N * W * 8),
                "aggregate": (lambda: dl.dlion_aggregate(packed, w.d, counts), w.N * W * 8 + 2 * w.d),
                "apply": (lambda: dl.dlion_apply(x, counts, w.N, w.mode, w.lr, w.lam), 10 * w.d),
                "aggregate_apply": (lambda: dl.dlion_aggregate_apply(x, packed, w.mode, w.lr, w.lam),
                                    w.N * W * 8 + 8 * w.d),
                "aggregate_encode": (lambda: dl.dlion_aggregate_encode(packed, w.d, w.mode, delta),
                                     w.N * W * 8 + planes * W * 8),
                "apply_encoded": (lambda: dl.dlion_apply_encoded(x, delta, w.N, w.mode, w.lr, w.lam),
                                  8 * w.d + planes * W * 8),
            }
            step, bytes_per_step = calls[entry]
            kernel = f"dlion_{entry} (packed rows and planes on 1 KB boundaries"
            ws_bytes = 0
            if entry != "worker_step":
                metric = f"coordinates/s (d per call of dlion_{entry})"
                units = w.d
    if w.g_dist != "packed_bernoulli":
        kernel += (f"; launches over 8 workers each, votes handed on in a {ws_bytes >> 20} MiB workspace)"
                   if ws_bytes else ")")
    torch.cuda.synchronize()

    kernel_ms, wall = timed(step, steps, warmup)
    achieved = bytes_per_step / (kernel_ms * 1e-3) / 1e9
    traffic, source = recorded_traffic(w.name, entry)
    rec = {
        "metric": metric,
        "value": units * steps / wall,
        "unit": metric.split(" ")[0],
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": wall / steps * 1e3,
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
            "traffic": traffic,                     # recorded by rocprofv3 earlier, not measured by this run
            "traffic_source": source,
            "kernel_ms": kernel_ms,                 # all launches of one step, HIP events on the launch stream
            "bytes_per_launch": bytes_per_step,     # algorithmic bytes of one step
            "bytes_per_update": bytes_per_step / units,
        },
    }
    if with_cpu_baseline and x is not None:
        rec["cpu_baseline"] = cpu_baseline(w, x, m, g)
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--entry", default="step", choices=ENTRIES,
                    help="measure one of the unfused calls on the workload's state instead of the fused step "
                         "(flat workloads with gradients; implies --headline-only --no-cpu-baseline)")
    ap.add_argument("--settle", type=float, default=SETTLE_S,
                    help="seconds to wait before the first allocation (see SETTLE_S)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="measure only --workload: no memory-rate ceilings, no short runs of the other workloads")
    ap.add_argument("--ceilings", action="store_true",
                    help="with --headline-only: still measure the memory-rate ceilings")
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
    time.sleep(max(0.0, args.settle))
    dev = "cuda:0"
    torch.cuda.set_device(0)
    dl.load_library()

    if args.entry != "step":
        cfg = wl.CONFIGS[args.workload]
        if cfg.shapes is not None or cfg.g_dist == "packed_bernoulli":
            print("--entry other than step needs a flat workload with gradients", file=sys.stderr)
            return 2
        args.headline_only = args.no_cpu_baseline = True
    rec = run_workload(args.workload, args.steps, args.warmup, dev, with_cpu_baseline=not args.no_cpu_baseline,
                       entry=args.entry)
    torch.cuda.empty_cache()
    out = {
        "metric": rec["metric"], "value": rec["value"], "unit": rec["unit"], "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": rec["config"], "roofline": rec["roofline"],
    }
    if "cpu_baseline" in rec:
        out["cpu_baseline"] = rec["cpu_baseline"]
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "launches": 5}
        del src, dst
    if args.headline_only and args.ceilings:
        del rec
        torch.cuda.empty_cache()
        out["roofline"].update(memory_ceilings(dev))
    if not args.headline_only:
        out["roofline"].update(memory_ceilings(dev))
        # every other workload in a process of its own (a fresh address space: what the headline's
        # 67 GB left behind in the allocator does not decide where their tensors land)
        import subprocess

        others = []
        del rec
        torch.cuda.empty_cache()
        for name in wl.CONFIGS:
            if name == args.workload:
                continue
            # about 0.1-0.2 s of timed work each
            n_steps = {"tiny": 2000, "gpt2s_avg8": 80, "vitb16_vote16": 50}.get(name, 8)
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", name, "--headline-only",
                   "--no-cpu-baseline", "--settle", str(SETTLE_CHILD_S), "--steps", str(n_steps),
                   "--warmup", str(max(2, n_steps // 10))]
            res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
            line = next((ln for ln in reversed(res.stdout.splitlines()) if ln.startswith("{")), None)
            if res.returncode != 0 or line is None:
                others.append({"workload": name, "error": (res.stderr or res.stdout)[-300:]})
                continue
            r = json.loads(line)
            others.append({"workload": name, "kernel": r["config"]["kernel"], "metric": r["metric"],
                           "value": r["value"], "ms_per_step": r["ms_per_step"],
                           "kernel_ms": r["roofline"]["kernel_ms"], "achieved_gbs": r["roofline"]["achieved"],
                           "frac": r["roofline"]["frac"], "steps": r["steps"]})
        out["workloads"] = others
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
