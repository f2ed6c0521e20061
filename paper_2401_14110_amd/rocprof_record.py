#!/usr/bin/env python3
"""Turns rocprofv3 runs of bench.py into the machine-readable counter record bench.py reports from.

bench.py measures time itself (HIP events); what only a profiler sees (HBM bytes, issued instructions) is
taken from separate rocprofv3 runs of the same command and stored in profiles/roofline_counters.json, keyed
by the workload and by the kernel's name, so that bench.py can attach the figures only to the kernel they were
measured on.  One record needs, all from the same build:

    cd /tmp && export TMPDIR=/tmp                       # on the GPU machine, repository root = $R
    python3 $R/bench.py <flags> --steps 5 --warmup 1 --no-cpu-baseline --dump-kernels $R/out/kernels.json
    rocprofv3 --kernel-trace --stats --output-format csv -d $R/out/prof_kt -- python3 $R/bench.py <flags> --steps 5 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES SQ_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_WAIT_INST_LDS \\
              --output-format csv -d $R/out/prof_sq -- python3 $R/bench.py <flags> --steps 1 --warmup 0 --no-cpu-baseline
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $R/out/prof_fetch -- python3 $R/bench.py <flags> --steps 1 --warmup 0 --no-cpu-baseline --copy-calibration
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $R/out/prof_write -- python3 $R/bench.py <flags> --steps 1 --warmup 0 --no-cpu-baseline --copy-calibration
    $R/paper_2401_14110_amd/valu_rate_probe > $R/out/valu_probe.txt

and then, anywhere (no GPU needed):

    python -m paper_2401_14110_amd.rocprof_record --kernels out/kernels.json --kt out/prof_kt \\
        --sq out/prof_sq --fetch out/prof_fetch --write out/prof_write \\
        --probe out/valu_probe.txt --probe-mix "mul|fma|and phased" --bench-flags "<flags>"

FETCH_SIZE / WRITE_SIZE are in KiB per dispatch and are scaled by what the same counter reads for a kernel of
known traffic in the same run: bench.py --copy-calibration ends with a torch add that reads 1 GiB and writes
1 GiB (the last dispatch of the run).  Replaces the record of the same workload key; other records are kept.
"""
import argparse
import csv
import glob
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "profiles", "roofline_counters.json")
GIB_KIB = float(1 << 20)


def short_name(full):
    """'void lba::lba_fast_mixed_kernel<32, 1, 0, 0>(lba::KParams)' -> 'lba_fast_mixed_kernel<32, 1, 0, 0>'"""
    m = re.match(r"^(?:void )?(?:lba::)?(lba_\w+(?:<[^()]*>)?)\(", full)
    return m.group(1) if m else None


def find_csv(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, d))
    return hits


def kernel_stats(d):
    """{short name: (calls, average ns)} summed over the processes of the run"""
    out = {}
    for path in find_csv(d, "_kernel_stats.csv"):
        for row in csv.DictReader(open(path)):
            n = short_name(row["Name"])
            if n:
                calls, tot = out.get(n, (0, 0.0))
                out[n] = (calls + int(row["Calls"]), tot + float(row["TotalDurationNs"]))
    return {n: (c, t / c) for n, (c, t) in out.items() if c}


def counters(d):
    """({short name: {counter: sum over dispatches}}, {short name: dispatches}, [(full name, counter, value) of the
    last dispatch])"""
    sums, disp, last, last_id = {}, {}, [], -1
    for path in find_csv(d, "_counter_collection.csv"):
        for row in csv.DictReader(open(path)):
            did = int(row["Dispatch_Id"])
            if did > last_id:
                last_id, last = did, []
            if did == last_id:
                last.append((row["Kernel_Name"], row["Counter_Name"], float(row["Counter_Value"])))
            n = short_name(row["Kernel_Name"])
            if n:
                c = sums.setdefault(n, {})
                c[row["Counter_Name"]] = c.get(row["Counter_Name"], 0.0) + float(row["Counter_Value"])
                disp.setdefault(n, set()).add(did)
    return sums, {n: len(v) for n, v in disp.items()}, last


def calibration(last, counter):
    """factor = true KiB / reported KiB for the final torch add of --copy-calibration (1 GiB read, 1 GiB written)"""
    vals = [v for (name, c, v) in last if c == counter and "at::native" in name]
    if not vals or vals[0] <= 0:
        raise SystemExit("the run for %s does not end with the torch calibration kernel (use --copy-calibration)" % counter)
    return GIB_KIB / vals[0], vals[0]


def probe_rates(path):
    """{'mul|fma|and phased': {...}} from the text the probe prints, at 4 waves per SIMD"""
    out = {}
    for line in open(path):
        m = re.match(r"^(.*?)\s+chains=\s*(\d+)\s+waves/SIMD=(\d+)\s+([\d.]+) SIMD-cycles/group \((\d+) instr\)\s+([\d.]+) lane-ops/clk/CU", line)
        if m and int(m.group(3)) == 4:
            rate = float(m.group(6))
            out[m.group(1).strip()] = {"lane_ops_per_clk_per_cu": rate, "lane_ops_per_s": 256 * rate * 2.4e9,
                                       "waves_per_simd": 4, "chains": int(m.group(2))}
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--kernels", required=True, help="bench.py --dump-kernels output")
    ap.add_argument("--kt", help="rocprofv3 --kernel-trace --stats output directory")
    ap.add_argument("--sq", help="directory of the SQ_* counter run (one step)")
    ap.add_argument("--fetch", help="directory of the FETCH_SIZE run (one step, --copy-calibration)")
    ap.add_argument("--write", help="directory of the WRITE_SIZE run (one step, --copy-calibration)")
    ap.add_argument("--probe", help="text printed by valu_rate_probe")
    ap.add_argument("--probe-mix", default=None, help="the probe's instruction mix that matches the kernels' inner loop")
    ap.add_argument("--bench-flags", default="", help="the flags bench.py was run with (recorded)")
    ap.add_argument("--commit", default=None, help="commit the runs were made from (default: git rev-parse of this checkout)")
    ap.add_argument("-o", "--out", default=OUT)
    args = ap.parse_args()

    dump = json.load(open(args.kernels))
    commit = args.commit or ""
    if not commit:
        try:
            commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
        except OSError:
            commit = ""
    rec = {"workload_key": dump["workload_key"], "bench_flags": args.bench_flags, "commit": commit or None, "kernels": {}}
    stats = kernel_stats(args.kt) if args.kt else {}
    sq, sq_n, _ = counters(args.sq) if args.sq else ({}, {}, [])
    fe, fe_n, fe_last = counters(args.fetch) if args.fetch else ({}, {}, [])
    wr, wr_n, wr_last = counters(args.write) if args.write else ({}, {}, [])
    f_fac = calibration(fe_last, "FETCH_SIZE") if args.fetch else (None, None)
    w_fac = calibration(wr_last, "WRITE_SIZE") if args.write else (None, None)
    for name, k in dump["kernels"].items():
        e = dict(k)
        if name in stats:
            e["trace_calls"], e["trace_avg_ns"] = stats[name]
        if name in sq:
            assert sq_n[name] == k["launches_per_step"], (name, sq_n[name], k["launches_per_step"])
            e["sq_per_step"] = sq[name]
            if "SQ_INSTS_VALU" in sq[name]:
                e["issued_valu_per_mac"] = sq[name]["SQ_INSTS_VALU"] * 64.0 / k["macs_per_step"]
            if "SQ_INSTS_SALU" in sq[name]:
                e["issued_salu_per_mac"] = sq[name]["SQ_INSTS_SALU"] * 64.0 / k["macs_per_step"]
        if name in fe and name in wr:
            assert fe_n[name] == wr_n[name] == k["launches_per_step"], (name, fe_n[name], wr_n[name])
            e["fetch_kib_per_step"], e["write_kib_per_step"] = fe[name]["FETCH_SIZE"], wr[name]["WRITE_SIZE"]
            e["fetch_factor"], e["write_factor"] = f_fac[0], w_fac[0]
            e["traffic_bytes_per_launch"] = 1024.0 * (fe[name]["FETCH_SIZE"] * f_fac[0] + wr[name]["WRITE_SIZE"] * w_fac[0]) / k["launches_per_step"]
            e["traffic_over_algorithmic"] = e["traffic_bytes_per_launch"] * k["launches_per_step"] / k["algorithmic_bytes_per_step"]
        if args.probe_mix:
            e["probe_mix"] = args.probe_mix
        rec["kernels"][name] = e
    if args.fetch:
        rec["calibration"] = {"kernel": "torch add over 2^28 floats: reads 1 GiB, writes 1 GiB",
                              "fetch_size_reported_kib": f_fac[1], "write_size_reported_kib": w_fac[1]}

    data = {"records": []}
    if os.path.exists(args.out):
        data = json.load(open(args.out))
    data["records"] = [r for r in data.get("records", []) if r.get("workload_key") != rec["workload_key"]] + [rec]
    if args.probe:
        data["valu_probe"] = probe_rates(args.probe)
    if args.probe_mix and args.probe_mix not in data.get("valu_probe", {}):
        raise SystemExit("probe mix %r is not in the probe output" % args.probe_mix)
    with open(args.out, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", args.out, "record", rec["workload_key"], "kernels", sorted(rec["kernels"]))


if __name__ == "__main__":
    sys.exit(main())
