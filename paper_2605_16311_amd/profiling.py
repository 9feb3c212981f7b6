"""rocprofv3 passes over bench.py and their text summaries.

    python3 paper_2605_16311_amd/profiling.py collect   --out DIR [--workload NAME] [--passes kt,fetch,write,mfma,peak]
    python3 paper_2605_16311_amd/profiling.py summarise --out DIR [--workload NAME] [--profiles profiles]

(run by path: the script imports neither the package nor torch.)  collect starts rocprofv3 as child
processes, each pass a run of its own with bench.py directly after "--"; this process itself never touches
the GPU.  Passes:
    kt     --kernel-trace --stats                     per-kernel durations
    fetch  --pmc FETCH_SIZE                           HBM bytes read per dispatch   (with a known-size copy)
    write  --pmc WRITE_SIZE                           HBM bytes written per dispatch
    mfma   --pmc SQ_VALU_MFMA_BUSY_CYCLES ...         matrix-core busy cycles, counted MFMA ops, clock
    cache  --pmc TCC_HIT_sum TCC_MISS_sum ...         L2 hits and misses, LDS bank conflicts (not in the default set)
    peak   mfma_peak                                  register-resident MFMA loop (no profiler)
summarise reads DIR and writes <profiles>/<workload>_kernel_trace.txt, _hbm_traffic.txt, _mfma_counters.txt,
_cache_counters.txt, mfma_loop_peak.txt and traffic.json (HBM bytes per launch by kernel class, read by bench.py).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
BENCH = os.path.join(ROOT, "bench.py")
MFMA_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16",
                 "SQ_INSTS_VALU_MFMA_MOPS_F16", "SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "GRBM_GUI_ACTIVE"]
CACHE_COUNTERS = ["TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum", "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE",
                  "TCP_PENDING_STALL_CYCLES_sum"]
SIMD_PER_XCD, XCDS = 128, 8          # 32 CUs x 4 SIMDs per XCD

# kernel classes of bench.py -> substring of the kernel name
CLASSES = {
    "sm_ns_gemm_kernel (Gram of Y)": ["sm_ns_gemm_kernel<0,"],
    "sm_ns_gemm_kernel (short-side recurrence)": ["sm_ns_gemm_kernel<3,", "sm_ns_gemm_kernel<2,"],
    "sm_ns_gemm_kernel (apply to Y)": ["sm_ns_gemm_kernel<1,"],
}


def bench_cmd(workload, steps, warmup, extra=()):
    return ["python3", BENCH, "--no-cpu-baseline", "--no-calibration", "--workload", workload, "--steps", str(steps),
            "--warmup", str(warmup), "--also", "", *extra]


def pass_commands(workload):
    return {
        "kt": ["rocprofv3", "--kernel-trace", "--stats", "-d", "{dir}", "-o", "bench", "--output-format", "csv", "--",
               *bench_cmd(workload, 10, 3)],
        "fetch": ["rocprofv3", "--pmc", "FETCH_SIZE", "-d", "{dir}", "-o", "bench", "--output-format", "csv", "--",
                  *bench_cmd(workload, 3, 1, ["--copy-calibration"])],
        "write": ["rocprofv3", "--pmc", "WRITE_SIZE", "-d", "{dir}", "-o", "bench", "--output-format", "csv", "--",
                  *bench_cmd(workload, 3, 1, ["--copy-calibration"])],
        "mfma": ["rocprofv3", "--pmc", *MFMA_COUNTERS, "-d", "{dir}", "-o", "bench", "--output-format", "csv", "--",
                 *bench_cmd(workload, 3, 1)],
        "cache": ["rocprofv3", "--pmc", *CACHE_COUNTERS, "-d", "{dir}", "-o", "bench", "--output-format", "csv", "--",
                  *bench_cmd(workload, 3, 1)],
        "peak": [os.path.join(HERE, "mfma_peak"), "200"],
    }


def collect(out, workload, passes):
    os.makedirs(out, exist_ok=True)
    env = dict(os.environ, TMPDIR="/tmp")
    cmds = pass_commands(workload)
    for name in passes:
        d = os.path.join(out, name)
        os.makedirs(d, exist_ok=True)
        cmd = [c.replace("{dir}", d) for c in cmds[name]]
        print("[profiling] pass", name, "->", d, flush=True)
        with open(os.path.join(d, "run.log"), "w") as log:
            try:
                r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=log, stderr=subprocess.STDOUT, timeout=400)
            except subprocess.TimeoutExpired:
                print(f"[profiling] pass {name} timed out; stopping", flush=True)
                return 124
        if r.returncode != 0:
            print(f"[profiling] pass {name} failed with {r.returncode}; see {d}/run.log; stopping", flush=True)
            return r.returncode
    return 0


def short(n):
    n = n.replace("void ", "").replace("(anonymous namespace)::", "").replace("sm_gemm::", "")
    return re.sub(r"\(.*", "", n)[:72]


def find(out, name, pattern):
    hits = glob.glob(os.path.join(out, name, "**", pattern), recursive=True)
    return hits[0] if hits else None


def printable(cmd):
    return " ".join(c if c else '""' for c in cmd).replace(ROOT + "/", "").replace("{dir}", "<out>")


def summarise_kt(out, workload, prof):
    f = find(out, "kt", "*kernel_stats.csv")
    if not f:
        return None
    rows = list(csv.DictReader(open(f)))
    lines = [f"rocprofv3 kernel trace, workload {workload}, one MI355X",
             "command (from /tmp, TMPDIR=/tmp):", "  " + printable(pass_commands(workload)["kt"]),
             "(3 warm-up + 10 timed steps, the same 10 with event taps on the GEMM launches, 10 with taps on every class,",
             " the standalone sign-pack / vote calls, then the captured and replayed steps of bench.py's graph_replay;",
             " bench_kernel_stats.csv, top rows)", "",
             "%-72s %6s %11s %10s %7s" % ("kernel", "calls", "total_ms", "avg_us", "pct")]
    avg = {}
    for r in rows:
        avg[r["Name"]] = (int(r["Calls"]), float(r["AverageNs"]) / 1e3)
    for r in rows[:14]:
        lines.append("%-72s %6s %11.3f %10.2f %7.2f" % (short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                                                        float(r["AverageNs"]) / 1e3, float(r["Percentage"])))
    lines += ["", "sm_ns_gemm_kernel<KIND, TILE>: KIND 0 = Gram of Y, 1 = apply to Y (the pre-vote launch also writes the packed",
              "  signs: there is no sign-pack kernel in the step), 3 = products of s x s matrices of the short-side recurrence",
              "  (2 = the same with whole-matrix storage); TILE = 256 before the vote, 128 after it on this workload.",
              "  bench.py's per-class avg_launch_ms is the mean over the launches of both tile sizes."]
    open(os.path.join(prof, f"{workload}_kernel_trace.txt"), "w").write("\n".join(lines) + "\n")
    return avg


def counter_means(path):
    """kernel name -> counter -> (dispatches, mean value per dispatch)."""
    acc = collections.defaultdict(lambda: collections.defaultdict(lambda: [0, 0.0]))
    for r in csv.DictReader(open(path)):
        a = acc[r["Kernel_Name"]][r["Counter_Name"]]
        a[0] += 1
        a[1] += float(r["Counter_Value"])
    return {k: {c: (v[0], v[1] / v[0]) for c, v in d.items()} for k, d in acc.items()}


def summarise_traffic(out, workload, prof):
    ff, fw = find(out, "fetch", "*counter_collection.csv"), find(out, "write", "*counter_collection.csv")
    if not ff or not fw:
        return
    fetch, write = counter_means(ff), counter_means(fw)

    def copy_mean(path, counter):
        vals = sorted(float(r["Counter_Value"]) for r in csv.DictReader(open(path))
                      if r["Kernel_Name"] == "__amd_rocclr_copyBuffer" and r["Counter_Name"] == counter)
        vals = vals[-3:]                                   # the three 1 GiB calibration copies are the largest
        return sum(vals) / len(vals)
    cf, cw = copy_mean(ff, "FETCH_SIZE"), copy_mean(fw, "WRITE_SIZE")
    sf, sw = 1048576.0 / cf, 1048576.0 / cw
    cmds = pass_commands(workload)
    lines = [f"HBM traffic per dispatch from rocprofv3 --pmc, workload {workload}, one MI355X",
             "commands (from /tmp, TMPDIR=/tmp), one counter per run:",
             "  " + printable(cmds["fetch"]), "  " + printable(cmds["write"]),
             "calibration: --copy-calibration runs three 1 GiB device-to-device copies (1 GiB read + 1 GiB written each);",
             "  FETCH_SIZE read %.0f KiB per copy  -> factor %.3f" % (cf, sf),
             "  WRITE_SIZE read %.0f KiB per copy -> factor %.3f" % (cw, sw), "",
             "%-64s %5s %14s %14s %13s" % ("kernel", "disp", "fetch_KiB_raw", "write_KiB_raw", "HBM_GB_scaled")]
    per_kernel = {}
    for k in fetch:
        if "sm_" not in k:
            continue
        n, fk = fetch[k].get("FETCH_SIZE", (0, 0.0))
        _, wk = write.get(k, {}).get("WRITE_SIZE", (0, 0.0))
        gb = (fk * sf + wk * sw) * 1024 / 1e9
        per_kernel[k] = (n, gb)
        lines.append("%-64s %5d %14.1f %14.1f %13.3f" % (short(k)[:64], n, fk, wk, gb))
    traffic = {}
    lines += ["", "per kernel class of bench.py (mean over the class's launches before and after the vote):"]
    for cname, pats in CLASSES.items():
        sel = [v for k, v in per_kernel.items() if any(p in k for p in pats)]
        n = sum(v[0] for v in sel)
        if not n:
            continue
        b = sum(v[0] * v[1] for v in sel) / n
        traffic[cname] = b * 1e9
        lines.append("  %-44s %7.3f GB per launch" % (cname, b))
    open(os.path.join(prof, f"{workload}_hbm_traffic.txt"), "w").write("\n".join(lines) + "\n")
    tpath = os.path.join(prof, "traffic.json")
    allt = {}
    if os.path.exists(tpath):
        try:
            allt = json.load(open(tpath))
        except ValueError:
            allt = {}
    allt[workload] = traffic
    allt["_note"] = ("HBM bytes per launch by kernel class: FETCH_SIZE x %.3f + WRITE_SIZE x %.3f "
                     "(see <workload>_hbm_traffic.txt)" % (sf, sw))
    json.dump(allt, open(tpath, "w"), indent=1)


def summarise_mfma(out, workload, prof, kt_avg):
    f = find(out, "mfma", "*counter_collection.csv")
    if not f:
        return
    m = counter_means(f)
    lines = [f"Matrix-core counters per dispatch from rocprofv3 --pmc, workload {workload}, one MI355X",
             "command (from /tmp, TMPDIR=/tmp):", "  " + printable(pass_commands(workload)["mfma"]),
             "columns: mean per dispatch.  mfma_busy = SQ_VALU_MFMA_BUSY_CYCLES (summed over SIMDs); gui = GRBM_GUI_ACTIVE (summed",
             "over the 8 XCDs); util = mfma_busy / (gui / 8 * 1024 SIMDs), the profiler's MfmaUtil: share of cycles the matrix",
             "pipe of a SIMD is busy at the clock the part ran at; flop = (MOPS_BF16 + MOPS_F16) * 512, the flops of the MFMA",
             "instructions issued (every tile the kernel computes, padding rows of ragged tiles included);",
             "clock = gui / 8 / kernel duration of the kernel-trace run (other run, same command line apart from --steps).", "",
             "%-40s %5s %12s %12s %7s %12s %10s %9s" % ("kernel", "disp", "mfma_busy", "gui", "util", "flop", "avg_us(kt)", "clock_GHz")]
    for k, d in sorted(m.items(), key=lambda kv: -kv[1].get("SQ_VALU_MFMA_BUSY_CYCLES", (0, 0))[1]):
        if "sm_ns_gemm" not in k:
            continue
        n, busy = d.get("SQ_VALU_MFMA_BUSY_CYCLES", (0, 0.0))
        gui = d.get("GRBM_GUI_ACTIVE", (0, 0.0))[1]
        flop = (d.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", (0, 0.0))[1] + d.get("SQ_INSTS_VALU_MFMA_MOPS_F16", (0, 0.0))[1]) * 512
        util = busy / (gui / XCDS * SIMD_PER_XCD * XCDS) if gui else 0.0
        us = kt_avg.get(k, (0, 0.0))[1] if kt_avg else 0.0
        clock = gui / XCDS / (us * 1e3) if us else 0.0
        lines.append("%-40s %5d %12.4g %12.4g %7.3f %12.4g %10.2f %9.2f" % (short(k)[:40], n, busy, gui, util, flop, us, clock))
        extra = {c: v[1] for c, v in d.items() if c in ("SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES")}
        lines.append("    " + "  ".join("%s %.4g" % kv for kv in sorted(extra.items())))
    open(os.path.join(prof, f"{workload}_mfma_counters.txt"), "w").write("\n".join(lines) + "\n")


def summarise_cache(out, workload, prof):
    f = find(out, "cache", "*counter_collection.csv")
    if not f:
        return
    m = counter_means(f)
    lines = [f"L2 and LDS counters per dispatch from rocprofv3 --pmc, workload {workload}, one MI355X",
             "command (from /tmp, TMPDIR=/tmp):", "  " + printable(pass_commands(workload)["cache"]),
             "columns: mean per dispatch.  l2_hit = TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum) over the 128-byte requests of all",
             "channels of the eight L2s; lds_conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE (cycles lost to bank conflicts",
             "per cycle the LDS spent on indexed accesses); tcp_pending = TCP_PENDING_STALL_CYCLES_sum (cycles a CU's vector L1",
             "could not take a request because of the requests it already had in flight).", "",
             "%-40s %5s %12s %12s %7s %12s %12s %9s %12s" % ("kernel", "disp", "l2_hit_req", "l2_miss_req", "l2_hit", "lds_conflict",
                                                          "lds_active", "conflict", "tcp_pending")]
    for k, d in sorted(m.items(), key=lambda kv: -kv[1].get("TCC_REQ_sum", (0, 0))[1]):
        if "sm_" not in k:
            continue
        n, hit = d.get("TCC_HIT_sum", (0, 0.0))
        miss = d.get("TCC_MISS_sum", (0, 0.0))[1]
        bc = d.get("SQ_LDS_BANK_CONFLICT", (0, 0.0))[1]
        act = d.get("SQ_LDS_IDX_ACTIVE", (0, 0.0))[1]
        pend = d.get("TCP_PENDING_STALL_CYCLES_sum", (0, 0.0))[1]
        lines.append("%-40s %5d %12.4g %12.4g %7.3f %12.4g %12.4g %9.3f %12.4g" % (
            short(k)[:40], n, hit, miss, hit / (hit + miss) if hit + miss else 0.0, bc, act, bc / act if act else 0.0, pend))
    open(os.path.join(prof, f"{workload}_cache_counters.txt"), "w").write("\n".join(lines) + "\n")


def summarise_peak(out, prof):
    f = os.path.join(out, "peak", "run.log")
    if not os.path.exists(f):
        return
    lines = ["Register-resident MFMA loop on one MI355X (no LDS, no memory traffic): the practical ceiling of the matrix cores",
             "command: paper_2605_16311_amd/mfma_peak 200    (built by __graft_entry__.build() from csrc/tools/mfma_peak.hip)", ""]
    lines += [ln.rstrip() for ln in open(f)]
    open(os.path.join(prof, "mfma_loop_peak.txt"), "w").write("\n".join(lines) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("cmd", choices=["collect", "summarise"])
    ap.add_argument("--out", required=True)
    ap.add_argument("--workload", default="nanogpt124m")
    ap.add_argument("--passes", default="kt,fetch,write,mfma,peak")
    ap.add_argument("--profiles", default=os.path.join(ROOT, "profiles"))
    a = ap.parse_args()
    if a.cmd == "collect":
        sys.exit(collect(os.path.abspath(a.out), a.workload, [p for p in a.passes.split(",") if p]))
    os.makedirs(a.profiles, exist_ok=True)
    kt_avg = summarise_kt(a.out, a.workload, a.profiles)
    summarise_traffic(a.out, a.workload, a.profiles)
    summarise_mfma(a.out, a.workload, a.profiles, kt_avg)
    summarise_cache(a.out, a.workload, a.profiles)
    summarise_peak(a.out, a.profiles)


if __name__ == "__main__":
    main()
