"""Turns rocprofv3 result databases of `bench.py` runs into the short text summaries kept under
profiles/ and into profiles/traffic.json (measured HBM bytes per launch of every kernel of this
library), which bench.py reports as `roofline.traffic`.

    python -m paper_2103_05288_amd.profile_summary --trace T.db --fetch F.db --write W.db \
        --bench-json trace_bench.json --out profiles

The three databases come from three runs of the same bench command (a kernel trace, a FETCH_SIZE
pass, a WRITE_SIZE pass; counters are collected in runs of their own).  FETCH_SIZE / WRITE_SIZE
count KiB per dispatch; what they read for a kernel is scaled by what the same counter reads for
the library's plain copy kernel, whose traffic is known (bench.py copies 1 GiB: 1 GiB read,
1 GiB written per launch).
"""
import argparse
import json
import os
import sqlite3

COPY_KERNEL = "disc_util_copy_k"
COPY_BYTES = 1 << 30          # bench.py's copy-ceiling measurement moves this much each way


def _ours(name: str) -> bool:
    return name.startswith("disc_")


def top_kernels(db):
    c = sqlite3.connect(db)
    rows = c.execute("select name, total_calls, total_duration, average, percentage from top_kernels").fetchall()
    c.close()
    return rows


def counter_per_kernel(db, counter):
    c = sqlite3.connect(db)
    rows = c.execute("select name, count(*), sum(counter_value) from pmc_events where counter_name = ? group by name",
                     (counter,)).fetchall()
    c.close()
    return {n: (k, s) for n, k, s in rows}


def short(name: str, n: int = 44) -> str:
    return name if len(name) <= n else name[:n - 1] + "~"


def next_rows_summary(args):
    """Kernel times and measured HBM bytes of the secondary workloads of bench.py (one large call
    each), next to the bytes of their inputs and outputs."""
    cmd_t = "rocprofv3 --kernel-trace --stats -d prof_out/nr_trace -o trace -- python3 bench.py --next-rows-only"
    cmd_c = "rocprofv3 --pmc {counter} -d prof_out/{dir} -o {dir} -- python3 bench.py --next-rows-only"
    rows = top_kernels(args.trace)
    avg_us = {name: avg for name, calls, tot, avg, pct in rows}
    lines = ["rocprofv3 kernel trace of bench.py's secondary workloads (one ~1 GB call each, repeated), MI355X",
             "command (from the repository root, after `cd /tmp && export TMPDIR=/tmp` on the GPU box):",
             "  " + cmd_t, "",
             "%-46s %8s %14s %12s %7s" % ("kernel", "calls", "total_us", "avg_us", "pct")]
    for name, calls, tot, avg, pct in rows:
        if _ours(name):
            lines.append("%-46s %8d %14.1f %12.3f %7.2f" % (short(name), calls, tot, avg, pct))
    b = json.load(open(args.bench_json)) if args.bench_json and os.path.exists(args.bench_json) else None
    if b:
        lines += ["", "bench.py's own figures from the same run (HIP events around ten calls, best of three):"]
        for k, v in b["next_rows"].items():
            lines.append("  %-28s dims %-34s %8.2f us  %7.1f GB/s of input + output bytes" % (k, v["dims"], v["us"], v["GBps"]))
    with open(os.path.join(args.out, "next_rows_kernel_trace.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")

    fetch = counter_per_kernel(args.fetch, "FETCH_SIZE")
    write = counter_per_kernel(args.write, "WRITE_SIZE")
    if COPY_KERNEL not in fetch or COPY_KERNEL not in write:
        raise SystemExit("the copy kernel is missing from the counter runs: no scale factors")
    f_scale = COPY_BYTES / (fetch[COPY_KERNEL][1] / fetch[COPY_KERNEL][0] * 1024.0)
    w_scale = COPY_BYTES / (write[COPY_KERNEL][1] / write[COPY_KERNEL][0] * 1024.0)
    per = {}
    for name in sorted(set(fetch) | set(write)):
        if not _ours(name) or name in ("disc_util_empty_k", COPY_KERNEL):
            continue
        nf, sf = fetch.get(name, (0, 0.0))
        nw, sw = write.get(name, (0, 0.0))
        per[name] = (sf * 1024.0 * f_scale / max(nf, 1), sw * 1024.0 * w_scale / max(nw, 1))
    lines = ["HBM traffic of bench.py's secondary workloads per kernel: rocprofv3 FETCH_SIZE and WRITE_SIZE, MI355X",
             "commands (one counter per run; from the repository root, after `cd /tmp && export TMPDIR=/tmp`):",
             "  " + cmd_c.format(counter="FETCH_SIZE", dir="nr_fetch"),
             "  " + cmd_c.format(counter="WRITE_SIZE", dir="nr_write"), "",
             "scale factors from the plain copy kernel %s (1 GiB each way per launch): FETCH_SIZE %.4f, WRITE_SIZE %.4f"
             % (COPY_KERNEL, f_scale, w_scale), "",
             "%-34s %16s %18s %12s" % ("kernel", "read MB/launch", "written MB/launch", "avg us")]
    for name, (rd, wr) in per.items():
        lines.append("%-34s %16.2f %18.2f %12.2f" % (name, rd / 1e6, wr / 1e6, avg_us.get(name, float("nan"))))
    if b:
        lines += ["", "per workload: bytes of the inputs and outputs (each once) against the measured bytes of its kernels:"]
        for k, v in b["next_rows"].items():
            mine = [n for n in per if any(n.startswith(p) for p in v.get("kernel_prefixes", []))] or \
                   [n for n in per if n in v.get("kernels", [])]
            meas = sum(per[n][0] + per[n][1] for n in mine)
            t = sum(avg_us.get(n, 0.0) for n in mine)
            if meas:
                lines.append("  %-28s algorithmic %9.2f MB  measured %9.2f MB  ratio %.3f  kernels %s (%.1f us in all: %.0f GB/s)"
                             % (k, v["io_bytes"] / 1e6, meas / 1e6, meas / v["io_bytes"], "+".join(mine), t, v["io_bytes"] / t / 1e3 if t else 0))
    with open(os.path.join(args.out, "next_rows_hbm_traffic.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines[-8:]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--bench-json", default="")
    ap.add_argument("--out", default="profiles")
    ap.add_argument("--trace-cmd", default="rocprofv3 --kernel-trace --stats -d prof_out/trace -o trace -- "
                                           "python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-gap-to-static --no-next-rows")
    ap.add_argument("--pmc-cmd", default="rocprofv3 --pmc {counter} -d prof_out/{dir} -o {dir} -- "
                                         "python3 bench.py --steps 1 --warmup 0 --no-cpu-baseline --no-gap-to-static --no-next-rows")
    ap.add_argument("--mode", default="sweep", choices=["sweep", "next_rows"],
                    help="next_rows: the three databases come from `bench.py --next-rows-only` runs; writes "
                         "next_rows_kernel_trace.txt and next_rows_hbm_traffic.txt and leaves traffic.json alone")
    args = ap.parse_args()
    os.makedirs(args.out, exist_ok=True)
    if args.mode == "next_rows":
        return next_rows_summary(args)

    # ---- kernel trace -------------------------------------------------------------------------
    rows = top_kernels(args.trace)
    total = sum(r[2] for r in rows)
    lines = ["rocprofv3 kernel trace of the whole bench step (C0-C4 dynamic-shape sweeps), MI355X",
             "command (from the repository root, after `cd /tmp && export TMPDIR=/tmp` on the GPU box; paths relative to the root):",
             "  " + args.trace_cmd,
             "",
             "%-46s %8s %14s %12s %7s" % ("kernel", "calls", "total_us", "avg_us", "pct")]
    for name, calls, tot, avg, pct in rows:
        if _ours(name) or pct >= 0.5:
            lines.append("%-46s %8d %14.1f %12.3f %7.2f" % (short(name), calls, tot, avg, pct))   # the view is in microseconds
    lines.append("")
    lines.append("all kernels in the process: %.1f ms; kernels of this library: %.1f ms"
                 % (total / 1e3, sum(r[2] for r in rows if _ours(r[0])) / 1e3))
    if args.bench_json and os.path.exists(args.bench_json):
        b = json.load(open(args.bench_json))
        r = b["roofline"]
        lines.append("")
        lines.append("bench.py's own line from the same run (HIP events around every call):")
        lines.append("  value %.1f GB/s (%.2f %% of 8 TB/s), copy ceiling %.1f GB/s (non-temporal copy %.1f GB/s)"
                     % (b["value"], b["pct_of_peak"], b["copy_ceiling_GBps"], b.get("copy_nt_ceiling_GBps", float("nan"))))
        lines.append("  roofline kernel %s: %d launches, avg %.2f us by HIP events, %.1f GB/s algorithmic"
                     % (r["kernel"], r["launches"], r["avg_launch_us"], r["achieved"]))
        for cfg, pc in b["per_config"].items():
            for k, v in pc["kernels"].items():
                lines.append("  %-3s %-60s launches %5d  avg %9.2f us  %7.1f GB/s" % (cfg, k, v["launches"], v["avg_us"], v["GBps"]))
    with open(os.path.join(args.out, "bench_sweep_kernel_trace.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")

    # ---- HBM traffic --------------------------------------------------------------------------
    fetch = counter_per_kernel(args.fetch, "FETCH_SIZE")
    write = counter_per_kernel(args.write, "WRITE_SIZE")
    if COPY_KERNEL not in fetch or COPY_KERNEL not in write:
        raise SystemExit("the copy kernel is missing from the counter runs: no scale factors")
    f_copy = fetch[COPY_KERNEL][1] / fetch[COPY_KERNEL][0] * 1024.0      # bytes per launch as counted
    w_copy = write[COPY_KERNEL][1] / write[COPY_KERNEL][0] * 1024.0
    f_scale = COPY_BYTES / f_copy
    w_scale = COPY_BYTES / w_copy
    traffic = {}
    lines = ["HBM traffic of the bench step per kernel: rocprofv3 FETCH_SIZE and WRITE_SIZE (KiB per dispatch), MI355X",
             "commands (one counter per run; from the repository root, after `cd /tmp && export TMPDIR=/tmp`):",
             "  " + args.pmc_cmd.format(counter="FETCH_SIZE", dir="fetch"),
             "  " + args.pmc_cmd.format(counter="WRITE_SIZE", dir="write"),
             "",
             "scale factors from the plain copy kernel %s (1 GiB read + 1 GiB written per launch):" % COPY_KERNEL,
             "  FETCH_SIZE reads %.1f MiB per launch  -> factor %.4f" % (f_copy / 2**20, f_scale),
             "  WRITE_SIZE reads %.1f MiB per launch  -> factor %.4f" % (w_copy / 2**20, w_scale),
             "",
             "%-34s %8s %16s %16s %16s" % ("kernel", "launches", "read MB/launch", "written MB/launch", "total MB/launch")]
    for name in sorted(set(fetch) | set(write)):
        if not _ours(name) or name == "disc_util_empty_k":
            continue
        nf, sf = fetch.get(name, (0, 0.0))
        nw, sw = write.get(name, (0, 0.0))
        rd = sf * 1024.0 * f_scale / max(nf, 1)
        wr = sw * 1024.0 * w_scale / max(nw, 1)
        traffic[name] = {"launches": int(max(nf, nw)), "read_bytes_per_launch": round(rd), "written_bytes_per_launch": round(wr),
                         "bytes_per_launch": round(rd + wr)}
        lines.append("%-34s %8d %16.2f %16.2f %16.2f" % (name, max(nf, nw), rd / 1e6, wr / 1e6, (rd + wr) / 1e6))
    if args.bench_json and os.path.exists(args.bench_json):
        b = json.load(open(args.bench_json))
        lines.append("")
        lines.append("algorithmic bytes per launch over the same sweeps (every operand and result once), from bench.py:")
        for cfg, pc in b["per_config"].items():
            for k, v in pc["kernels"].items():
                names = k.split("+")
                alg = v["GBps"] * 1e9 * v["avg_us"] * 1e-6
                meas = sum(traffic[n]["bytes_per_launch"] for n in names if n in traffic)
                if meas:
                    lines.append("  %-3s %-60s algorithmic %10.2f MB  measured %10.2f MB  ratio %.3f"
                                 % (cfg, k, alg / 1e6, meas / 1e6, meas / alg))
    with open(os.path.join(args.out, "bench_sweep_hbm_traffic.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    with open(os.path.join(args.out, "traffic.json"), "w") as f:
        json.dump(traffic, f, indent=1, sort_keys=True)
    print("\n".join(lines[-12:]))


if __name__ == "__main__":
    main()
