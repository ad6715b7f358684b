"""Writes a short text summary (``profiles/<kernel>_<workload>.md``) from rocprofv3 result databases.

Usage (after the rocprofv3 runs named in the summary it writes)::

    python -m paper_2404_00438_amd.profile_summary --workload gpt350m_vote32 --kernel step_kernel \
        --title "fused dlion_step kernel" --stats S.db --fetch F.db --write W.db [--busy B.db] \
        --trace-steps 23 --pmc-steps 6 --out profiles/dlion_step_gpt350m_vote32.md

``S.db`` comes from ``rocprofv3 --kernel-trace --stats``, ``F.db`` / ``W.db`` from ``--pmc FETCH_SIZE`` /
``--pmc WRITE_SIZE`` and ``B.db`` from ``--pmc MeanOccupancyPerCU VALUBusy``, each over
``bench.py --workload W [--entry E] --headline-only --no-cpu-baseline --copy-calibration``.  The counters are scaled
against the 1 GiB device copies that ``--copy-calibration`` adds to the run.  ``--trace-steps`` /
``--pmc-steps`` are steps + warm-up steps of the respective runs, i.e. how many steps' launches the
databases hold.  Only reads the databases; nothing here runs on a GPU.
"""
from __future__ import annotations

import argparse
import sqlite3

GIB_KIB = 1048576.0


def rows(db, sql):
    con = sqlite3.connect(db)
    try:
        return con.execute(sql).fetchall()
    finally:
        con.close()


def kernel_stats(db):
    return rows(db, "select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                    "from kernels group by name order by sum(end-start) desc")


def counters(db):
    return rows(db, "select kernel_name, counter_name, count(*), avg(value), min(value), max(value), "
                    "max(vgpr_count), max(accum_vgpr_count), max(sgpr_count), max(lds_block_size), "
                    "max(workgroup_size), max(grid_size) from counters_collection "
                    "group by kernel_name, counter_name order by avg(value) desc")


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--entry", default="step", help="what bench.py measured (its --entry)")
    ap.add_argument("--kernel", required=True, help="substring of the kernel name(s) the summary is about")
    ap.add_argument("--title", required=True)
    ap.add_argument("--stats", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--busy")
    ap.add_argument("--trace-steps", type=int, required=True)
    ap.add_argument("--pmc-steps", type=int, required=True)
    ap.add_argument("--bench-args", default="", help="what followed bench.py on the kernel-trace command line")
    ap.add_argument("--bench-log", help="stdout of the kernel-trace run: its JSON line gives the algorithmic bytes "
                                        "and, if the run had --ceilings, the memory-rate ceilings")
    ap.add_argument("--out", required=True)
    a = ap.parse_args(argv)

    k = kernel_stats(a.stats)
    total = sum(r[2] for r in k)
    f, w = counters(a.fetch), counters(a.write)
    fks = [r for r in f if a.kernel in r[0] and r[1] == "FETCH_SIZE"]
    wks = [r for r in w if a.kernel in r[0] and r[1] == "WRITE_SIZE"]
    fc = [r for r in f if "copyBuffer" in r[0]][0]
    wc = [r for r in w if "copyBuffer" in r[0]][0]
    f_scale, w_scale = GIB_KIB / fc[5], GIB_KIB / wc[5]     # the largest copies are the 1 GiB calibration copies
    fetch_bytes = sum(r[2] * r[3] for r in fks) / a.pmc_steps * f_scale * 1024
    write_bytes = sum(r[2] * r[3] for r in wks) / a.pmc_steps * w_scale * 1024
    launches = sum(r[2] for r in fks) / a.pmc_steps
    ks = [r for r in k if a.kernel in r[0]]
    bench = (f"python3 $R/bench.py --workload {a.workload}" + (f" --entry {a.entry}" if a.entry != "step" else "") +
             " --headline-only --no-cpu-baseline --copy-calibration")

    L = [f"# rocprofv3 summary: {a.title}, workload `{a.workload}`\n",
         "Commands (run from /tmp with TMPDIR=/tmp, repository root = $R; each rocprofv3 run on its own):\n", "```",
         (f"rocprofv3 --kernel-trace --stats -d $T/stats -o stats -- {bench} {a.bench_args}".rstrip() +
          (" > $T/stats.log" if a.bench_log else "")),
         f"rocprofv3 --pmc FETCH_SIZE -d $T/fetch -o fetch -- {bench} --steps 5 --warmup 1",
         f"rocprofv3 --pmc WRITE_SIZE -d $T/write -o write -- {bench} --steps 5 --warmup 1"]
    if a.busy:
        L.append(f"rocprofv3 --pmc MeanOccupancyPerCU VALUBusy -d $T/busy -o busy -- {bench} --steps 5 --warmup 1")
    L.append(f"python3 -m paper_2404_00438_amd.profile_summary --workload {a.workload} "
             + (f"--entry {a.entry} " if a.entry != "step" else "") + f"--kernel {a.kernel} "
             f"--title \"{a.title}\" --stats $T/stats/stats_results.db --fetch $T/fetch/fetch_results.db "
             f"--write $T/write/write_results.db" + (" --busy $T/busy/busy_results.db" if a.busy else "") +
             f" --trace-steps {a.trace_steps} --pmc-steps {a.pmc_steps}" +
             (" --bench-log $T/stats.log" if a.bench_log else "") + " --out profiles/<this file>")
    L += ["```\n", "## Kernel trace (--kernel-trace --stats): the kernel in question, then the top kernels by total time\n",
          "| kernel | calls | total ms | avg us | min us | max us | % |", "|---|---|---|---|---|---|---|"]
    for r in ks + [r for r in k if r not in ks][:6]:
        L.append(f"| `{r[0][:110]}` | {r[1]} | {r[2] / 1e6:.3f} | {r[3] / 1e3:.2f} | {r[4] / 1e3:.2f} | "
                 f"{r[5] / 1e3:.2f} | {100 * r[2] / total:.1f} |")
    L.append("\nRows other than the library's kernels are input generation (torch random draws) and the calibration copy; "
             "membench_kernel is the memory-rate probe behind the ceilings below.\n")
    L.append("## Launch shape (from the counter run's dispatch records)\n")
    for r in fks:
        L.append(f"- `{r[0][:100]}`: grid up to {r[11]} work-items, workgroup {r[10]}, VGPRs {r[6]}, AGPRs {r[7]}, "
                 f"SGPRs {r[8]}, LDS reserved per workgroup {r[9]} B (caps the resident waves per compute unit)")
    L.append("\n## HBM traffic (--pmc FETCH_SIZE, then --pmc WRITE_SIZE; counter values are per dispatch)\n")
    L += ["| kernel | counter | dispatches | avg | min | max |", "|---|---|---|---|---|---|"]
    for r in (*fks, fc, *wks, wc):
        L.append(f"| `{r[0][:80]}` | {r[1]} | {r[2]} | {r[3]:.1f} | {r[4]:.1f} | {r[5]:.1f} |")
    L.append("\n(The copy rows include torch's own small device copies; the calibration uses the largest ones, the 1 GiB copies.)\n")
    L.append(f"Calibration: the plain device copy moves exactly 1 GiB in and 1 GiB out (1,048,576 KiB each way) per "
             f"launch, so the scale factors are FETCH_SIZE x{f_scale:.4f} and WRITE_SIZE x{w_scale:.4f} to KiB.\n")
    if a.busy:
        b = [r for r in counters(a.busy) if a.kernel in r[0]]
        L.append("## Occupancy and vector-ALU activity (--pmc MeanOccupancyPerCU VALUBusy, per dispatch)\n")
        L += ["| kernel | counter | dispatches | avg | min | max |", "|---|---|---|---|---|---|"]
        for r in b:
            L.append(f"| `{r[0][:80]}` | {r[1]} | {r[2]} | {r[3]:.2f} | {r[4]:.2f} | {r[5]:.2f} |")
        L.append("\nMeanOccupancyPerCU = resident waves per compute unit averaged over the kernel's run; VALUBusy = % of "
                 "cycles in which a compute unit issues a vector-ALU instruction.\n")
    L.append(f"One step of this workload = {launches:g} launch(es) of the kernel; figures below are per step "
             f"(dispatches x avg, summed over the kernel's variants, / steps).\n")
    L.append(f"- kernel time per step (kernel trace): {sum(r[2] for r in ks) / a.trace_steps / 1e6:.4f} ms")
    L.append(f"- fetched per step: {fetch_bytes:.0f} B")
    L.append(f"- written per step: {write_bytes:.0f} B")
    L.append(f"- traffic_bytes_per_launch: {fetch_bytes + write_bytes:.0f}")
    if a.bench_log:
        import json

        with open(a.bench_log) as fh:
            line = next(ln for ln in reversed(fh.read().splitlines()) if ln.startswith("{"))
        r = json.loads(line)["roofline"]
        ms = sum(x[2] for x in ks) / a.trace_steps / 1e6
        gbs = r["bytes_per_launch"] / ms / 1e6
        L.append(f"- algorithmic bytes per step: {r['bytes_per_launch']} (traffic / algorithmic = "
                 f"{(fetch_bytes + write_bytes) / r['bytes_per_launch']:.4f})")
        L.append(f"- achieved (algorithmic bytes / kernel-trace time): {gbs:.1f} GB/s = {100 * gbs / 8000:.1f} % of the "
                 f"8 TB/s peak")
        keys = [("copy_ceiling_gbs", "plain copy"), ("read_ceiling_gbs", "read only (8 rows per wave)"),
                ("mix16to1_ceiling_gbs", "16 rows read per row written (the byte mix of counting 256 streams)")]
        if any(k in r for k, _ in keys):
            L.append("\n## Memory-rate ceilings measured in the same run (dlion_membench: no arithmetic, best of several launch shapes)\n")
            L += ["| probe | GB/s | % of peak | this kernel / probe |", "|---|---|---|---|"]
            for k, label in keys:
                if k in r:
                    L.append(f"| {label} | {r[k]:.0f} | {100 * r[k] / 8000:.1f} | {gbs / r[k]:.3f} |")
    with open(a.out, "w") as fh:
        fh.write("\n".join(L) + "\n")
    print("\n".join(L))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
