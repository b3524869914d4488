"""Reduces rocprofv3 CSV output of `bench.py` to the short text summaries kept under profiles/.

    python -m paper_2101_01321_amd.rocprof_summary stats   <dir-of-kernel-trace-run>  [--title TEXT] [--command TEXT]
    python -m paper_2101_01321_amd.rocprof_summary traffic <fetch-run-dir> <write-run-dir>         -> .txt on stdout, .json with --json PATH
    python -m paper_2101_01321_amd.rocprof_summary counters <pmc-run-dir> [<pmc-run-dir> ...]

A run directory is what `rocprofv3 ... -d <dir> -o bench -- python3 bench.py ...` wrote (bench_kernel_stats.csv for
--kernel-trace --stats, bench_counter_collection.csv for --pmc).  Only kernels of this library (namespace ibert::) are kept;
copy kernels of the runtime are used for the FETCH_SIZE / WRITE_SIZE calibration (bench.py --copy-calibration).
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import sys


def _find(run_dir, suffix):
    hits = sorted(glob.glob(os.path.join(run_dir, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, run_dir))
    return hits[0]


def short(name):
    name = name.replace("void ibert::", "").replace("ibert::", "")
    return re.sub(r"\((GemmArgs|[A-Za-z_:]+Args|.*)\)$", "", name)


def step_of(name):
    """Which step of the layer a kernel name belongs to (for the reader; from the template arguments)."""
    if name.startswith("attention"):
        return "S2-4"
    if name.startswith("softmax"):
        return "S3"
    if name.startswith("isqrt"):
        return "isqrt"
    if name.startswith("layernorm"):
        a = [x.strip() for x in name[name.index("<") + 1:name.rindex(">")].split(",")]
        return "EMB" if len(a) > 3 and a[3] == "true" else "LN"
    if name.startswith("gelu_kernel"):
        return "hGELU" if name.endswith("true>") else "GELU"
    m = re.match(r"gemm_nt_mfma_kernel<(\d+), (\d+), (\d+), (\d+), (\w+), (\d), (\w+), (\w+), (\w+), (\d+), (\d+)>", name)
    if not m:
        return "?"
    bm, bn, bk, ring, i8, km, tw, dma, gelu, nw, nld = m.groups()
    if gelu == "true":
        return "S7+8"
    if i8 == "true":
        return "S1"
    return "S5/S9"


def cmd_stats(args):
    rows = [r for r in csv.DictReader(open(_find(args.run, "kernel_stats.csv"))) if "ibert::" in r["Name"]]
    tot = sum(float(r["TotalDurationNs"]) for r in rows)
    out = []
    if args.title:
        out.append(args.title)
    if args.command:
        out.append("command (from /tmp, TMPDIR=/tmp):")
        out.append("  " + args.command)
    out.append("")
    out.append("%-78s %-6s %6s %11s %8s %6s %8s %8s" % ("kernel (ibert::)", "step", "calls", "total_us", "avg_us", "pct", "min_us", "max_us"))
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"])):
        n = short(r["Name"])
        out.append("%-78s %-6s %6s %11.1f %8.2f %6.2f %8.2f %8.2f" % (
            n, step_of(n), r["Calls"], float(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3,
            100 * float(r["TotalDurationNs"]) / tot, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))
    print("\n".join(out))


def _counter_means(run_dir):
    """{kernel short name: {counter: mean per dispatch}}, plus the same for the runtime's copy kernel."""
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(_find(run_dir, "counter_collection.csv"))):
        k = r["Kernel_Name"]
        if "ibert::" in k:
            key = short(k)
        elif "copyBuffer" in k:
            key = "__copy__"
        else:
            continue
        agg.setdefault(key, collections.OrderedDict()).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    return {k: {c: (sum(v) / len(v), max(v), len(v)) for c, v in cs.items()} for k, cs in agg.items()}


def cmd_traffic(args):
    fetch, write = _counter_means(args.fetch), _counter_means(args.write)
    cal_f = fetch["__copy__"]["FETCH_SIZE"][1]          # KiB the counter reads for the 256 MiB copy (largest dispatch)
    cal_w = write["__copy__"]["WRITE_SIZE"][1]
    fs, ws = 262144.0 / cal_f, 262144.0 / cal_w
    out = ["HBM-side traffic per launch (rocprofv3 --pmc, one counter per run) -- bench.py, one MI355X"]
    if args.command:
        out += ["commands (from /tmp, TMPDIR=/tmp):", "  " + args.command.replace("COUNTER", "FETCH_SIZE"),
                "  " + args.command.replace("COUNTER", "WRITE_SIZE")]
    out.append("calibration: a plain 256 MiB device-to-device copy (262144 KiB read, 262144 KiB written) reads FETCH_SIZE = %.0f KiB and" % cal_f)
    out.append("WRITE_SIZE = %.0f KiB per dispatch -> FETCH_SIZE is scaled by %.2f, WRITE_SIZE by %.2f below." % (cal_w, fs, ws))
    out.append("")
    out.append("%-78s %-6s %10s %11s" % ("kernel", "step", "read MB", "written MB"))
    js = {"config": args.config, "fetch_scale": round(fs, 3), "write_scale": round(ws, 3), "kernel_sources_sha256": args.digest,
          "kernels": {}}
    for k in fetch:
        if k == "__copy__" or k not in write:
            continue
        rd, wr = fetch[k]["FETCH_SIZE"][0] * 1024 * fs, write[k]["WRITE_SIZE"][0] * 1024 * ws
        out.append("%-78s %-6s %10.2f %11.2f" % (k, step_of(k), rd / 1e6, wr / 1e6))
        label = k if k.startswith("gemm") else re.sub(r"^(\w+)<.*$", r"\1", k) + ("<embedding>" if step_of(k) == "EMB" else "") + \
            ("<h-GELU>" if step_of(k) == "hGELU" else "")
        js["kernels"][label] = {"read": round(rd), "written": round(wr)}
    print("\n".join(out))
    if args.json:
        json.dump(js, open(args.json, "w"), indent=1)


def cmd_counters(args):
    merged = collections.OrderedDict()
    for d in args.runs:
        for k, cs in _counter_means(d).items():
            if k == "__copy__":
                continue
            merged.setdefault(k, collections.OrderedDict()).update({c: v[0] for c, v in cs.items()})
    out = []
    if args.title:
        out.append(args.title)
    if args.command:
        out += ["commands (from /tmp, TMPDIR=/tmp; one run per counter group):", "  " + args.command]
    out.append("Counter values are means per dispatch, summed over the chip (256 compute units, 1024 SIMDs) by the profiler.")
    out.append("SQ_BUSY_CU_CYCLES and SQ_VALU_MFMA_BUSY_CYCLES count clock cycles; SQ_WAVE_CYCLES and SQ_WAIT_* count 4-cycle units.  Derived:")
    out.append("  cu_cyc      = SQ_BUSY_CU_CYCLES / 256: busy cycles of the average compute unit per launch")
    out.append("  mfma_busy   = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES): share of the SIMD-cycles of busy compute units in which the")
    out.append("                MFMA pipe works (cyc/mfma = pipe cycles per MFMA instruction; 16 for v_mfma_i32_16x16x64_i8)")
    out.append("  valu_slots  = (SQ_INSTS_VALU - SQ_INSTS_MFMA) / SQ_BUSY_CU_CYCLES: vector-ALU instructions x 4 issue cycles per SIMD-cycle; a lower")
    out.append("                bound of the ALU pipe's occupancy, because the 64-bit multiply-adds of requantization hold it for 8 or more")
    out.append("  lds_active  = SQ_LDS_IDX_ACTIVE / SQ_BUSY_CU_CYCLES (a 16-byte-per-lane read counts about 4 here and takes 8 cycles at the")
    out.append("                measured 128 B/clk, so the LDS pipe is occupied for about twice this share)")
    out.append("  lds_conf    = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE: LDS cycles lost to bank conflicts per active LDS cycle")
    out.append("  wait_any    = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of a wavefront's life spent waiting for outstanding memory or LDS data")
    out.append("  wait_lds    = SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES")
    out.append("  icache_miss = SQC_ICACHE_MISSES / SQC_ICACHE_REQ")
    out.append("")

    def ratio(c, a, b, scale=1.0, sub=None):
        if a not in c or b not in c or not c[b]:
            return "       -"
        return "%8.3f" % (scale * (c[a] - (c.get(sub, 0.0) if sub else 0.0)) / c[b])
    hdr = "%-74s %-6s %8s %9s %8s %10s %10s %8s %8s %8s %11s"
    out.append(hdr % ("kernel", "step", "cu_cyc", "mfma_busy", "cyc/mfma", "valu_slots", "lds_active", "lds_conf", "wait_any", "wait_lds", "icache_miss"))
    for k, c in merged.items():
        out.append(hdr % (
            k[:74], step_of(k), "%8.0f" % (c["SQ_BUSY_CU_CYCLES"] / 256) if "SQ_BUSY_CU_CYCLES" in c else "-",
            ratio(c, "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", 0.25), ratio(c, "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_MFMA"),
            ratio(c, "SQ_INSTS_VALU", "SQ_BUSY_CU_CYCLES", 1.0, "SQ_INSTS_MFMA"), ratio(c, "SQ_LDS_IDX_ACTIVE", "SQ_BUSY_CU_CYCLES"),
            ratio(c, "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE"),
            ratio(c, "SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"), ratio(c, "SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES"),
            ratio(c, "SQC_ICACHE_MISSES", "SQC_ICACHE_REQ")))
    out.append("")
    out.append("raw means per dispatch:")
    names = []
    for c in merged.values():
        for n in c:
            if n not in names:
                names.append(n)
    for k, c in merged.items():
        out.append("  " + k)
        out.append("     " + "  ".join("%s=%.4g" % (n, c[n]) for n in names if n in c))
    print("\n".join(out))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("run")
    s.add_argument("--title", default="")
    s.add_argument("--command", default="")
    t = sub.add_parser("traffic")
    t.add_argument("fetch")
    t.add_argument("write")
    t.add_argument("--command", default="")
    t.add_argument("--config", default="base_b32")
    t.add_argument("--digest", default="")
    t.add_argument("--json", default="")
    c = sub.add_parser("counters")
    c.add_argument("runs", nargs="+")
    c.add_argument("--title", default="")
    c.add_argument("--command", default="")
    args = ap.parse_args()
    {"stats": cmd_stats, "traffic": cmd_traffic, "counters": cmd_counters}[args.what](args)


if __name__ == "__main__":
    main()
