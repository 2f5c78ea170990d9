"""Turns the rocprofv3 output of the benchmark into the short summaries kept under profiles/.

Inputs (directories written by rocprofv3, see the commands in the summary's header):
    <prof>/stats/bench_kernel_stats.csv              rocprofv3 --kernel-trace --stats of bench.py
    <prof>/pmc_FETCH_SIZE, <prof>/pmc_WRITE_SIZE     rocprofv3 --pmc of bench.py
    <prof>/copy_FETCH_SIZE, <prof>/copy_WRITE_SIZE   the same counters on copy_probe.py (1 GiB copies)

Outputs:
    profiles/<kernel>_<workload>.md   per-kernel time, counter readings, calibration, traffic
    profiles/hbm_traffic.json         HBM bytes per chain-kernel launch, keyed by workload and
                                      tagged with the digest of the kernel sources (bench.py
                                      quotes the number only while the sources are unchanged)

    python -m paper_1708_04801_amd.profile_summary out/prof dense_logistic
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

COPY_BYTES = 1024 * (1 << 20)


def _counters(directory):
    agg = collections.defaultdict(list)
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        with open(path) as fh:
            for r in csv.DictReader(fh):
                agg[(r["Kernel_Name"], r["Counter_Name"])].append(float(r["Counter_Value"]))
    return agg


def _mean(agg, kernel_part, counter):
    vals = [v for (k, c), vs in agg.items() if kernel_part in k and c == counter for v in vs]
    return sum(vals) / len(vals) if vals else None


def main():
    prof, workload = sys.argv[1], sys.argv[2]
    from bench import kernel_source_digest

    stats = []
    with open(os.path.join(prof, "stats", "bench_kernel_stats.csv")) as fh:
        for r in csv.DictReader(fh):
            stats.append(r)
    chain = next(r for r in stats if "chain_" in r["Name"])
    kernel_name = chain["Name"]
    short = kernel_name.split("<")[0].split("::")[-1].split("(")[0].replace("void ", "").strip()

    bench_line = None
    with open(os.path.join(prof, "stats_stdout.log")) as fh:
        for ln in fh:
            if ln.startswith('{"metric"'):
                bench_line = json.loads(ln)

    factors, readings = {}, {}
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        copy_val = _mean(_counters(os.path.join(prof, f"copy_{ctr}")), "copyBuffer", ctr)
        factors[ctr] = COPY_BYTES / copy_val              # bytes per counter unit
        readings[ctr] = _mean(_counters(os.path.join(prof, f"pmc_{ctr}")), "chain_", ctr)
    traffic = readings["FETCH_SIZE"] * factors["FETCH_SIZE"] + readings["WRITE_SIZE"] * factors["WRITE_SIZE"]

    cfg, roof = bench_line["config"], bench_line["roofline"]
    algo = roof["bytes_per_sample_update"] * cfg["sample_updates_per_step"]
    lines = [
        f"# {short} on {workload}: rocprofv3 summary",
        "",
        "Commands (run from /tmp on the MI355X box, repository at $R):",
        "",
        f"    rocprofv3 --kernel-trace --stats -d out/stats -o bench --output-format csv -- python3 $R/bench.py --no-cpu-baseline --workload {workload}",
        f"    rocprofv3 --pmc FETCH_SIZE -d out/pmc_FETCH_SIZE -o bench --output-format csv -- python3 $R/bench.py --no-cpu-baseline --steps 2 --warmup 1 --workload {workload}",
        f"    rocprofv3 --pmc WRITE_SIZE -d out/pmc_WRITE_SIZE -o bench --output-format csv -- python3 $R/bench.py --no-cpu-baseline --steps 2 --warmup 1 --workload {workload}",
        "    rocprofv3 --pmc FETCH_SIZE -d out/copy_FETCH_SIZE -o copy --output-format csv -- python3 $R/paper_1708_04801_amd/copy_probe.py",
        "    rocprofv3 --pmc WRITE_SIZE -d out/copy_WRITE_SIZE -o copy --output-format csv -- python3 $R/paper_1708_04801_amd/copy_probe.py",
        "",
        f"Workload: {json.dumps(cfg)}",
        "",
        "## Kernel time (--kernel-trace --stats)",
        "",
        "| kernel | calls | average (ms) | min (ms) | max (ms) | share |",
        "|---|---|---|---|---|---|",
    ]
    for r in stats:
        if "wpsgd::" in r["Name"]:
            nm = r["Name"].split("(")[0].replace("void ", "")
            lines.append(f"| `{nm}` | {r['Calls']} | {float(r['AverageNs']) / 1e6:.4f} | "
                         f"{float(r['MinNs']) / 1e6:.4f} | {float(r['MaxNs']) / 1e6:.4f} | {float(r['Percentage']):.2f} % |")
    lines += [
        "",
        f"bench.py's own HIP-event figure for the chain kernel in the same run: {roof['kernel_ms']:.4f} ms "
        f"(rocprofv3 average {float(chain['AverageNs']) / 1e6:.4f} ms).",
        "",
        "## HBM traffic of the chain kernel (--pmc, one counter per run)",
        "",
        "| counter | reading per dispatch | 1 GiB copy reads | bytes per unit | bytes per dispatch |",
        "|---|---|---|---|---|",
    ]
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        lines.append(f"| {ctr} | {readings[ctr]:.1f} | {COPY_BYTES / factors[ctr]:.1f} | {factors[ctr]:.1f} | "
                     f"{readings[ctr] * factors[ctr]:.4g} |")
    lines += [
        "",
        f"HBM traffic per launch: {traffic:.5g} bytes; algorithmic bytes per launch "
        f"({roof['bytes_per_sample_update']:.0f} B x {cfg['sample_updates_per_step']} sample-updates): {algo:.5g}; "
        f"ratio {traffic / algo:.4f}.",
        "",
        f"Achieved (algorithmic) bandwidth {roof['achieved']:.1f} GB/s = {100 * roof['frac']:.2f} % of the 8 TB/s peak.",
    ]
    ceil = roof.get("k_compute_units_streaming_alone")
    if ceil:
        lines += [
            "",
            f"What {ceil['workgroups']} compute units draw from HBM on their own (`stream_rows_kernel`, no arithmetic): "
            f"{ceil['streaming_GBps']:.1f} GB/s; chains are alive {100 * ceil['alive_fraction']:.1f} % of the kernel's "
            f"duration on average, which would allow {ceil['attainable_GBps']:.1f} GB/s; the chain kernel reaches "
            f"{100 * ceil['frac_of_attainable']:.1f} % of that (more than all of it where idle compute units take part: helper "
            "workgroups that pull the rows into L2 ahead of the chains, or chains cut into column slices).",
        ]
    if "us_per_step_longest_chain" in roof:
        lines += ["", f"Longest chain: {roof['longest_chain_steps']} steps, {roof['us_per_step_longest_chain']:.3f} us per step "
                      "(the launch lasts as long as its longest chain)."]
    lines.append(f"\nKernel source digest: {kernel_source_digest()}")
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", f"{short}_{workload}.md"), "w") as fh:
        fh.write("\n".join(lines) + "\n")

    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    table = {}
    if os.path.exists(path):
        with open(path) as fh:
            table = json.load(fh)
    table[workload] = {"hbm_bytes_per_launch": traffic, "kernel": kernel_name,
                       "kernel_source_digest": kernel_source_digest(),
                       "fetch_bytes_per_unit": factors["FETCH_SIZE"], "write_bytes_per_unit": factors["WRITE_SIZE"]}
    with open(path, "w") as fh:
        json.dump(table, fh, indent=1, sort_keys=True)
    print("\n".join(lines))


if __name__ == "__main__":
    main()
