"""Profile one benchmark configuration with rocprofv3 and write its summary.

    python -m paper_2501_11779_amd.rocprof_summary --workload c4 [--sq] [--tag NAME]
                                                   [--bench-args="--paged ..."] [--out DIR]
    python -m paper_2501_11779_amd.rocprof_summary --ceiling [--out DIR]

Runs, each as its own rocprofv3 process around `python3 bench.py ...` (counters never share a run
with a trace): the kernel trace with statistics, one FETCH_SIZE pass and one WRITE_SIZE pass (both
with bench.py's 1 GiB calibration copy, the known-size kernel the readings are scaled by), and with
--sq two passes of shader counters.  Writes DIR/gh_decode_attention_<tag>.md and, for the
library's default launch of a workload (no --bench-args), that workload's entry of
DIR/traffic.json -- the file bench.py takes `roofline.traffic` from.  DIR defaults to profiles/;
raw rocprofv3 output goes to a temporary directory and is deleted.

This is a measurement tool: it starts child processes and parses their CSV files, and touches
neither the GPU nor the library itself.
"""
import argparse
import csv
import glob
import json
import os
import re
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")
CONFIG_OF = {"c1": "configs[0]", "c2": "configs[1]", "c3": "configs[2]", "c4": "configs[3]",
             "c5": "configs[4]"}
SQ_PASSES = (
    "SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_VMEM "
    "SQ_WAIT_INST_ANY SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VMEM_RD",
    "GRBM_GUI_ACTIVE SQ_WAVES SQ_INSTS_VMEM_WR SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_INSTS_VALU "
    "SQ_INSTS_MFMA SQ_WAIT_ANY",
)
COPY_KIB = 1048576.0


def rocprof(work, name, options, bench_args, limit_s=300):
    """One rocprofv3 run; returns (rows of every CSV it wrote by suffix, bench.py's stderr)."""
    out_dir = os.path.join(work, name)
    cmd = ["rocprofv3", *options, "--output-format", "csv", "-d", out_dir, "-o", name, "--",
           sys.executable, BENCH, *bench_args]
    env = dict(os.environ, TMPDIR="/tmp")
    print("+ " + " ".join(cmd), flush=True)
    res = subprocess.run(["timeout", "-s", "KILL", str(limit_s), *cmd], cwd="/tmp", env=env,
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr[-4000:])
        raise SystemExit(f"rocprofv3 run '{name}' failed with status {res.returncode}")
    tables = {}
    for path in glob.glob(os.path.join(out_dir, "**", "*.csv"), recursive=True):
        with open(path, newline="") as fh:
            tables[os.path.basename(path)[len(name) + 1:-4]] = list(csv.DictReader(fh))
    shown = " ".join(["rocprofv3", *options, "--output-format", "csv", "-d", f"/tmp/{name}", "-o",
                      name, "--", "python3", "$R/bench.py", *bench_args])
    return tables, res.stderr, shown


def per_kernel(rows, counter):
    agg = {}
    for r in rows:
        if r["Counter_Name"] == counter:
            agg.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return agg


def short(name):
    return name.replace("void ", "")


def summarise_workload(args, work):
    wl, tag = args.workload, args.tag or args.workload
    extra = args.bench_args.split() if args.bench_args else []
    base = ["--workload", wl, *extra, "--no-cpu-baseline", "--no-other-workloads"]
    out = [f"# rocprofv3 summary: Tier-2 attention step, workload {tag} ({CONFIG_OF[wl]}"
           f"{', ' + args.bench_args if args.bench_args else ''}), MI355X (gfx950)\n",
           "Written by `python -m paper_2501_11779_amd.rocprof_summary --workload " + wl
           + (f' --tag {tag} --bench-args="{args.bench_args}"' if args.bench_args else "")
           + (" --sq" if args.sq else "") + "`, which ran (from /tmp, `TMPDIR=/tmp`, `$R` = "
           "repository root):\n"]
    kt, log, c1 = rocprof(work, f"kt_{tag}", ["--kernel-trace", "--stats"],
                          [*base, "--steps", "50", "--warmup", "10"])
    cal = [*base, "--steps", "5", "--warmup", "2", "--pmc-calibration"]
    fe, _, c2 = rocprof(work, f"fetch_{tag}", ["--pmc", "FETCH_SIZE"], cal)
    wr, _, c3 = rocprof(work, f"write_{tag}", ["--pmc", "WRITE_SIZE"], cal)
    out += ["```", c1, c2, c3, "```\n"]

    out += ["## Kernel durations (`--kernel-trace --stats`, this library's kernels only)\n",
            "| kernel | calls | average (us) | min (us) | max (us) | stddev (us) |", "|---|---|---|---|---|---|"]
    attn_avg_us = None
    for r in kt["kernel_stats"]:
        if "gh::" in r["Name"]:
            out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | "
                       f"{float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f} | "
                       f"{float(r['StdDev']) / 1e3:.2f} |")
            if "attn_" in r["Name"]:
                attn_avg_us = float(r["AverageNs"]) / 1e3
    line = [ln for ln in log.splitlines() if ln.startswith("step ")]
    if line:
        out.append(f"\nbench.py's own HIP-event reading in the same run: `{line[-1]}`\n")

    out += ["## HBM traffic counters (`--pmc`, KiB per dispatch)\n",
            "| kernel | counter | dispatches | mean KiB | scaled bytes (mean) |", "|---|---|---|---|---|"]
    fetch = per_kernel(fe["counter_collection"], "FETCH_SIZE")
    write = per_kernel(wr["counter_collection"], "WRITE_SIZE")
    # the calibration copy: the runtime's buffer-copy kernel whose dispatch writes 1 GiB
    cal_kernel = next(k for k, v in write.items()
                      if "copyBuffer" in k and abs(max(v) - COPY_KIB) < 0.02 * COPY_KIB)
    w_fac = max(write[cal_kernel]) / COPY_KIB
    f_fac = max(fetch[cal_kernel]) / COPY_KIB
    out.append(f"| `{short(cal_kernel)[:60]}` (calibration: plain 1 GiB device copy) | FETCH_SIZE | 1 | "
               f"{max(fetch[cal_kernel]):.1f} | factor {f_fac:.4f} of the 1048576 KiB read |")
    out.append(f"| same | WRITE_SIZE | 1 | {max(write[cal_kernel]):.1f} | factor {w_fac:.4f} of the "
               f"1048576 KiB written |")
    scaled = {}
    for counter, agg, fac in (("FETCH_SIZE", fetch, f_fac), ("WRITE_SIZE", write, w_fac)):
        for k, v in agg.items():
            if "gh::" in k:
                mean = sum(v) / len(v)
                scaled[(k, counter)] = mean * 1024 / fac
                out.append(f"| `{short(k)}` | {counter} | {len(v)} | {mean:.1f} | "
                           f"{mean * 1024 / fac / 1e6:.1f} MB |")
    attn = next(k for k in fetch if "gh::attn_" in k)
    traffic = scaled[(attn, "FETCH_SIZE")] + scaled[(attn, "WRITE_SIZE")]
    out.append(f"\nAttention kernel HBM traffic per launch (fetch + write, scaled): "
               f"**{traffic / 1e9:.4f} GB**\n")

    if args.sq:
        out += ["## Shader counters of the attention kernel (`--pmc`, two passes, mean per dispatch, "
                "summed over the chip)\n", "```"]
        sq = {}
        for i, counters in enumerate(SQ_PASSES):
            t, _, c = rocprof(work, f"sq{i + 1}_{tag}", ["--pmc", *counters.split()],
                              [*base, "--steps", "5", "--warmup", "2"])
            out.append(c)
            for r in t["counter_collection"]:
                if "gh::attn_" in r["Kernel_Name"]:
                    sq.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        out += ["```\n", "| counter | mean per dispatch |", "|---|---|"]
        m = {k: sum(v) / len(v) for k, v in sq.items()}
        out += [f"| {k} | {m[k]:.0f} |" for k in sorted(m)]
        cyc = m["GRBM_GUI_ACTIVE"] / 8
        out += ["", "Read together (wave-level counters tick once per four cycles; 1024 SIMDs, 8 XCDs):\n",
                f"- {m['SQ_WAVES']:.0f} waves; {m['SQ_INSTS_MFMA'] / 1e6:.2f} M matrix instructions, "
                f"{m['SQ_INSTS_VMEM_RD'] / 1e6:.2f} M vector loads, {m['SQ_INSTS_VMEM_WR'] / 1e3:.1f} K "
                f"vector stores, {m['SQ_INSTS_LDS'] / 1e6:.2f} M LDS instructions "
                f"({m['SQ_LDS_BANK_CONFLICT']:.0f} conflict cycles) per launch.",
                f"- matrix pipe busy {m['SQ_VALU_MFMA_BUSY_CYCLES'] / 1e6:.0f} M SIMD-cycles = "
                f"{m['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024 / cyc * 100:.1f}% of the kernel's cycles per "
                f"SIMD (GRBM_GUI_ACTIVE / 8 XCDs = {cyc / 1e6:.2f} M cycles).",
                f"- of the waves' resident time (SQ_WAVE_CYCLES), "
                f"{m['SQ_WAIT_INST_ANY'] / m['SQ_WAVE_CYCLES'] * 100:.0f}% is spent waiting to issue "
                f"(SQ_WAIT_INST_ANY) and {m['SQ_ACTIVE_INST_VALU'] / m['SQ_WAVE_CYCLES'] * 100:.0f}% "
                f"executing vector arithmetic (SQ_ACTIVE_INST_VALU).",
                f"- resident waves per SIMD on average: "
                f"{m['SQ_WAVE_CYCLES'] * 4 / 1024 / cyc:.2f} (SQ_WAVE_CYCLES x 4 / 1024 SIMDs / kernel "
                f"cycles) -- below the launch's waves per SIMD when waves finish at different times.\n"]

    os.makedirs(args.out, exist_ok=True)
    name = f"gh_decode_attention_{tag}.md"
    with open(os.path.join(args.out, name), "w") as fh:
        fh.write("\n".join(out) + "\n")
    print(f"wrote {os.path.join(args.out, name)}: attention {attn_avg_us} us, traffic {traffic / 1e9:.4f} GB")
    if not args.bench_args:
        path = os.path.join(args.out, "traffic.json")
        table = {}
        if os.path.exists(path):
            with open(path) as fh:
                table = json.load(fh)
        table[wl] = {"attention_bytes_per_launch": round(traffic),
                     "fetch_bytes": round(scaled[(attn, "FETCH_SIZE")]),
                     "write_bytes": round(scaled[(attn, "WRITE_SIZE")]),
                     "fetch_factor": f_fac, "write_factor": w_fac, "kernel": short(attn),
                     "attention_avg_us_kernel_trace": attn_avg_us, "summary": f"profiles/{name}"}
        with open(path, "w") as fh:
            json.dump(table, fh, indent=1, sort_keys=True)
            fh.write("\n")


def summarise_ceiling(args, work):
    kt, log, cmd = rocprof(work, "kt_ceiling", ["--kernel-trace", "--stats"],
                           ["--ceiling", "--steps", "10", "--warmup", "3"])
    out = ["# rocprofv3 summary: streaming-read probe (include/gh_probe.h), MI355X (gfx950)\n",
           "The rate the memory system gives the attention kernel's access shape when nothing else is "
           "in the way: 2048 waves, each reading its own contiguous share of 8 GiB in 16 KiB tiles of "
           "whole 128-byte lines, one to three tiles in flight, non-temporal loads; alone, and with a 4 KiB "
           "store per wave every 64 or 16 tiles in each store policy; reads alone also with 1024 waves, "
           "one per SIMD.  A measurement aid; the "
           "roofline peak stays the published 8 TB/s.\n",
           "Written by `python -m paper_2501_11779_amd.rocprof_summary --ceiling`, which ran (from "
           "/tmp, `TMPDIR=/tmp`, `$R` = repository root):\n", "```", cmd, "```\n",
           "## Kernel durations (`--kernel-trace --stats`)\n",
           "| kernel | calls | average (us) | min (us) | GB/s at the average | % of 8 TB/s |",
           "|---|---|---|---|---|---|"]
    for r in kt["kernel_stats"]:
        if "probe_stream_kernel" in r["Name"]:
            avg = float(r["AverageNs"])
            rate = (8 << 30) / avg
            label = re.search(r"probe_stream_kernel<[^>]*>", r["Name"]).group(0)
            out.append(f"| `{label}` | {r['Calls']} | {avg / 1e3:.2f} | "
                       f"{float(r['MinNs']) / 1e3:.2f} | {rate:.0f} | {rate / 80:.1f} |")
    out.append("\n(`<-1>`: no stores, the average taken over the runs with 2048 and with 1024 waves; `<0>` plain, `<1>` non-temporal, `<2>` write-through stores, the "
               "average taken over both store spacings.)\n")
    out.append("bench.py's own HIP-event readings in the same run, per case:\n\n```")
    out += [ln for ln in log.splitlines() if ln.startswith("stream probe")]
    out.append("```")
    os.makedirs(args.out, exist_ok=True)
    with open(os.path.join(args.out, "stream_read_ceiling.md"), "w") as fh:
        fh.write("\n".join(out) + "\n")
    print(f"wrote {os.path.join(args.out, 'stream_read_ceiling.md')}")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", choices=sorted(CONFIG_OF))
    ap.add_argument("--tag", default="", help="name of the summary (default: the workload)")
    ap.add_argument("--bench-args", default="", help="further bench.py arguments, e.g. '--paged'")
    ap.add_argument("--sq", action="store_true", help="also collect shader counters (two more runs)")
    ap.add_argument("--ceiling", action="store_true", help="profile bench.py --ceiling instead")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    args = ap.parse_args()
    if not args.ceiling and not args.workload:
        ap.error("--workload or --ceiling")
    if args.bench_args and not args.tag:
        ap.error("--bench-args needs a --tag for the summary's name")
    work = tempfile.mkdtemp(prefix="gh_rocprof_", dir="/tmp")
    try:
        (summarise_ceiling if args.ceiling else summarise_workload)(args, work)
    finally:
        shutil.rmtree(work, ignore_errors=True)


if __name__ == "__main__":
    main()
