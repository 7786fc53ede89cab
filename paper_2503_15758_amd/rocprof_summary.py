"""rocprofv3 passes over bench.py and the text summaries kept under profiles/.

Two commands (run from the repository root, on the MI355X machine):

  python -m paper_2503_15758_amd.rocprof_summary collect --workload c3 --dir raw/prof_c3
      runs bench.py five times under rocprofv3 (kernel trace; FETCH_SIZE; WRITE_SIZE; two passes of
      SQ activity counters), each pass in a run of its own, and leaves the raw CSV output, bench.py's
      JSON line and its launch log in <dir>/<pass>/.

  python -m paper_2503_15758_amd.rocprof_summary tables --workload c3 --dir raw/prof_c3 --out profiles
      turns that raw output into profiles/<workload>_kernel_trace.txt, _hbm_traffic.txt and
      _utilisation.txt.  The traffic file ends with machine-readable lines that bench.py reads
      (`traffic_bytes <call> <bytes>`), stamped with the hash of the kernel sources they were
      measured on, so that a table older than the kernels is visible.

How a launch is told apart: bench.py --launch-log writes, in launch order, which call of the step
every kernel launch of the process belongs to; the CSV rows of the library's kernels, sorted by
start time, are matched to that list one to one (the counts must agree).

HBM counters: FETCH_SIZE / WRITE_SIZE count in KiB per dispatch on some units and over-count on
others; both are scaled by what the same counter reads for the library's plain copy kernel of
known size (bench.py --copy-probe, 1 GiB), launched in the same profiler run.
"""
import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)

PASSES = {
    "kt": ["--kernel-trace", "--stats"],
    "fetch": ["--pmc", "FETCH_SIZE"],
    "write": ["--pmc", "WRITE_SIZE"],
    "util1": ["--pmc", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE",
              "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_BUSY_CU_CYCLES", "GRBM_GUI_ACTIVE"],
    "util2": ["--pmc", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_VALU_MFMA_COEXEC_CYCLES", "SQ_ACTIVE_INST_VALU",
              "SQ_ACTIVE_INST_LDS", "SQ_WAIT_INST_LDS", "SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES", "GRBM_GUI_ACTIVE"],
}
# optional passes (collect --memory-path): where vector-memory instructions wait
MEMORY_PASSES = {
    "vmem": ["--pmc", "SQ_INSTS_VMEM_WR", "SQ_INST_CYCLES_VMEM_WR", "SQ_VMEM_WR_TA_DATA_FIFO_FULL",
             "SQ_VMEM_TA_ADDR_FIFO_FULL", "SQ_INSTS_VMEM_RD", "SQ_INST_CYCLES_VMEM_RD", "SQ_WAVE_CYCLES", "GRBM_GUI_ACTIVE"],
    "tc": ["--pmc", "TCP_TCC_WRITE_REQ_LATENCY_sum", "TCP_TCC_WRITE_REQ_sum", "TCP_PENDING_STALL_CYCLES_sum",
           "TCC_EA0_WRREQ_STALL_sum", "TCC_EA0_WRREQ_sum", "TCC_TOO_MANY_EA_WRREQS_STALL_sum", "GRBM_GUI_ACTIVE"],
}
BENCH_STEPS = {"kt": ("10", "3"), "fetch": ("2", "1"), "write": ("2", "1"), "util1": ("2", "1"), "util2": ("2", "1"),
               "vmem": ("2", "1"), "tc": ("2", "1")}


def source_hash():
    """sha256 over the kernel sources and headers (what the measured numbers depend on)."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")) + glob.glob(os.path.join(PKG, "csrc", "*.hpp")) +
                   [os.path.join(ROOT, "include", "a2d.h")])
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def git_head():
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True,
                              check=True).stdout.strip()
    except Exception:
        return "unknown"


def pass_command(workload, name, out_dir, extra):
    steps, warm = BENCH_STEPS[name]
    cmd = ["rocprofv3"] + (PASSES.get(name) or MEMORY_PASSES[name]) + ["--output-format", "csv", "-d", out_dir, "-o", "bench", "--",
                                          "python3", "bench.py", "--workload", workload, "--steps", steps,
                                          "--warmup", warm, "--no-cpu-baseline", "--no-extras", "--copy-probe",
                                          "--launch-log", os.path.join(out_dir, "launches.json")] + list(extra)
    return cmd


def collect(args):
    os.makedirs(args.dir, exist_ok=True)
    env = dict(os.environ, TMPDIR="/tmp")
    for name in list(PASSES) + (list(MEMORY_PASSES) if args.memory_path else []):
        out_dir = os.path.join(args.dir, name)
        os.makedirs(out_dir, exist_ok=True)
        cmd = pass_command(args.workload, name, out_dir, args.bench_args.split())
        print("[rocprof_summary] pass %s: %s" % (name, " ".join(cmd)), flush=True)
        with open(os.path.join(out_dir, "bench.json"), "w") as fo, open(os.path.join(out_dir, "stderr.txt"), "w") as fe:
            r = subprocess.run(["timeout", "-s", "KILL", "420"] + cmd, cwd=ROOT, env=env, stdout=fo, stderr=fe)
        print("[rocprof_summary] pass %s ended with status %d" % (name, r.returncode), flush=True)
        if r.returncode != 0:
            sys.exit("pass %s failed; see %s" % (name, os.path.join(out_dir, "stderr.txt")))
    with open(os.path.join(args.dir, "stamp.json"), "w") as f:
        json.dump({"git_head": git_head(), "source_sha256": source_hash(), "workload": args.workload,
                   "bench_args": args.bench_args.split()}, f)


# ----------------------------------------------------------------------------- parsing
def short_name(k):
    m = re.match(r"_ZN3a2d12_GLOBAL__N_1\d+([a-z_0-9]+kernel)", k) or \
        re.search(r"a2d::\(anonymous namespace\)::([a-z_0-9]+kernel)", k)
    return m.group(1) if m else None


def _find(out_dir, pattern):
    hits = glob.glob(os.path.join(out_dir, "**", pattern), recursive=True)
    if not hits:
        sys.exit("no %s under %s" % (pattern, out_dir))
    return sorted(hits)[0]


def _bench_line(out_dir):
    for line in open(os.path.join(out_dir, "bench.json")):
        if line.startswith("{"):
            return line.strip()
    return ""


def kernel_rows(out_dir):
    """the library's kernel launches of a kernel-trace pass in start order, each joined with its
    launch-log entry: (kernel, call, phase, duration_us, grid, wg)"""
    rows = list(csv.DictReader(open(_find(out_dir, "*kernel_trace.csv"))))
    rows = [r for r in rows if short_name(r["Kernel_Name"])]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    log = json.load(open(os.path.join(out_dir, "launches.json")))
    if len(rows) != len(log):
        sys.exit("%s: %d library kernels in the trace, %d in the launch log" % (out_dir, len(rows), len(log)))
    out = []
    for r, e in zip(rows, log):
        k = short_name(r["Kernel_Name"])
        if k != e["kernel"]:
            sys.exit("%s: trace has %s where the launch log has %s" % (out_dir, k, e["kernel"]))
        out.append((k, e["call"], e["phase"], (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3,
                    r.get("Grid_Size_X", r.get("Grid_Size", "")), r.get("Workgroup_Size_X", r.get("Workgroup_Size", ""))))
    return out


def counter_rows(out_dir):
    """{counter: [(kernel, call, phase, value)] in dispatch order} of a --pmc pass"""
    rows = list(csv.DictReader(open(_find(out_dir, "*counter_collection.csv"))))
    rows = [r for r in rows if short_name(r["Kernel_Name"])]
    per_counter = collections.defaultdict(list)
    for r in rows:
        per_counter[r["Counter_Name"]].append(r)
    log = json.load(open(os.path.join(out_dir, "launches.json")))
    out = {}
    for ctr, rs in per_counter.items():
        # one row per dispatch and counter (several if the counter is reported per instance: summed)
        by_dispatch = collections.OrderedDict()
        for r in sorted(rs, key=lambda r: int(r["Dispatch_Id"])):
            d = by_dispatch.setdefault(int(r["Dispatch_Id"]), [short_name(r["Kernel_Name"]), 0.0])
            d[1] += float(r["Counter_Value"])
        vals = list(by_dispatch.values())
        if len(vals) != len(log):
            sys.exit("%s: %d dispatches carry %s, the launch log has %d" % (out_dir, len(vals), ctr, len(log)))
        out[ctr] = [(k, e["call"], e["phase"], v) for (k, v), e in zip(vals, log) if k == e["kernel"]]
        if len(out[ctr]) != len(log):
            sys.exit("%s: kernel names of %s do not follow the launch log" % (out_dir, ctr))
    return out


def _avg(v):
    return sum(v) / len(v) if v else float("nan")


def tables(args):
    wl = args.workload
    name = args.name or wl                      # prefix of the files written
    stamp = json.load(open(os.path.join(args.dir, "stamp.json")))
    if stamp["git_head"] == "unknown" and stamp["source_sha256"] == source_hash():
        stamp["git_head"] = git_head() + " or later (same kernel sources)"   # the box that measured had no .git
    os.makedirs(args.out, exist_ok=True)
    cmd = lambda name: "  " + " ".join(pass_command(wl, name, os.path.join(args.dir, name), stamp.get("bench_args", [])))
    head = ["workload %s, kernel sources %s, git head %s" % (wl, stamp["source_sha256"], stamp["git_head"]),
            "made by: python -m paper_2503_15758_amd.rocprof_summary collect --workload %s --dir %s   (then `tables`)"
            % (wl, args.dir), ""]

    # ---- kernel trace
    kt = kernel_rows(os.path.join(args.dir, "kt"))
    groups = collections.OrderedDict()
    for k, call, phase, us, grid, wg in kt:
        if phase == "setup":
            continue
        groups.setdefault((k, call, grid, wg), []).append(us)
    out = ["rocprofv3 kernel-trace summary of bench.py"] + head + ["command:", cmd("kt"), "",
           "Per kernel and call of the step (warm-up and timed steps; set-up launches left out), microseconds:", "",
           "%-22s %-18s %10s %5s %6s %10s %10s %10s" % ("kernel", "call", "grid", "wg", "calls", "avg_us", "min_us", "max_us")]
    for (k, call, grid, wg), v in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
        out.append("%-22s %-18s %10s %5s %6d %10.1f %10.1f %10.1f" % (k, call, grid, wg, len(v), _avg(v), min(v), max(v)))
    out += ["", "bench.py line of the same run (per-kernel times there come from HIP events on the launch stream):",
            _bench_line(os.path.join(args.dir, "kt"))]
    open(os.path.join(args.out, "%s_kernel_trace.txt" % name), "w").write("\n".join(out) + "\n")

    # ---- HBM traffic
    fetch = counter_rows(os.path.join(args.dir, "fetch"))["FETCH_SIZE"]
    write = counter_rows(os.path.join(args.dir, "write"))["WRITE_SIZE"]
    probe_kib = (1 << 30) / 1024.0
    pf = [v for k, c, p, v in fetch if k == "copy_probe_kernel"]
    pw = [v for k, c, p, v in write if k == "copy_probe_kernel"]
    fs, ws = probe_kib / _avg(pf), probe_kib / _avg(pw)
    per = collections.OrderedDict()
    for (k, call, phase, v), (_, _, _, wv) in zip(fetch, write):
        if phase == "setup" or k == "copy_probe_kernel":
            continue
        d = per.setdefault((call, k), [[], []])
        d[0].append(v * fs * 1024.0)
        d[1].append(wv * ws * 1024.0)
    out = ["HBM traffic per launch from rocprofv3 PMC counters over bench.py"] + head + \
          ["commands (one counter per run):", cmd("fetch"), cmd("write"), "",
           "Scale factors from the library's copy kernel (a2d_copy_probe, 1 GiB read and 1 GiB written per launch):",
           "  FETCH_SIZE reads %.0f KiB -> factor %.3f;  WRITE_SIZE reads %.0f KiB -> factor %.3f" % (_avg(pf), fs, _avg(pw), ws),
           "", "Per launch, averaged over the steps, scaled, MiB:", "",
           "%-18s %-22s %12s %12s" % ("call", "kernel", "read MiB", "written MiB")]
    per_call = collections.OrderedDict()
    for (call, k), (rv, wv) in per.items():
        out.append("%-18s %-22s %12.1f %12.1f" % (call, k, _avg(rv) / 2 ** 20, _avg(wv) / 2 ** 20))
        per_call[call] = per_call.get(call, 0.0) + _avg(rv) + _avg(wv)
    out += ["", "# machine-readable (bench.py reads the lines below; bytes per launch of the whole call / of one kernel)",
            "source_sha256 %s" % stamp["source_sha256"], "git_head %s" % stamp["git_head"]]
    for call, b in per_call.items():
        out.append("traffic_bytes %s %d" % (call, round(b)))
    for (call, k), (rv, wv) in per.items():
        out.append("traffic_bytes %s/%s %d" % (call, k, round(_avg(rv) + _avg(wv))))
    open(os.path.join(args.out, "%s_hbm_traffic.txt" % name), "w").write("\n".join(out) + "\n")

    # ---- utilisation
    u1 = counter_rows(os.path.join(args.dir, "util1"))
    u2 = counter_rows(os.path.join(args.dir, "util2"))
    kt_us = collections.OrderedDict()
    for k, call, phase, us, grid, wg in kt:
        if phase != "setup":
            kt_us.setdefault((call, k), []).append(us)

    def mean_of(rows):
        d = collections.OrderedDict()
        for k, call, phase, v in rows:
            if phase != "setup" and k != "copy_probe_kernel":
                d.setdefault((call, k), []).append(v)
        return {key: _avg(v) for key, v in d.items()}

    m1 = {c: mean_of(r) for c, r in u1.items()}
    m2 = {c: mean_of(r) for c, r in u2.items()}
    out = ["MFMA / vector-ALU / LDS activity per launch from rocprofv3 PMC counters over bench.py"] + head + \
          ["commands (two runs, at most 8 SQ counters each):", cmd("util1"), cmd("util2"), "",
           "cycles = GRBM_GUI_ACTIVE / 8 XCDs; GHz = cycles / kernel-trace duration; MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES /",
           "(1024 SIMDs x cycles); co-exec = SQ_VALU_MFMA_COEXEC_CYCLES on the same base (MFMA unit and vector ALU of a SIMD both",
           "working); VALU = 4 x SQ_ACTIVE_INST_VALU / (1024 x cycles); LDS = SQ_LDS_IDX_ACTIVE / (256 CUs x cycles); conflicts =",
           "SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE; wait any / wait LDS = SQ_WAIT_INST_ANY / SQ_WAIT_INST_LDS over SQ_WAVE_CYCLES;",
           "MFMA TFLOP = 512 x SQ_INSTS_VALU_MFMA_MOPS_BF16 (executed, recomputation included).", "",
           "%-18s %-20s %8s %6s %9s %8s %6s %6s %9s %9s %9s %10s" % ("call", "kernel", "time us", "GHz", "MFMA busy", "co-exec",
                                                                  "VALU", "LDS", "conflicts", "wait any", "wait LDS", "MFMA TFLOP")]
    for key in m1.get("GRBM_GUI_ACTIVE", {}):
        call, k = key
        cyc = m1["GRBM_GUI_ACTIVE"][key] / 8.0
        cyc2 = m2["GRBM_GUI_ACTIVE"].get(key, float("nan")) / 8.0
        us = _avg(kt_us.get(key, []))
        g = lambda m, c: m.get(c, {}).get(key, float("nan"))
        lds_act = g(m1, "SQ_LDS_IDX_ACTIVE")
        out.append("%-18s %-20s %8.0f %6.2f %8.1f%% %7.1f%% %5.1f%% %5.1f%% %8.1f%% %8.1f%% %8.1f%% %10.3f" % (
            call, k, us, cyc / us / 1e3 if us == us else float("nan"),
            100 * g(m1, "SQ_VALU_MFMA_BUSY_CYCLES") / (1024 * cyc),
            100 * g(m2, "SQ_VALU_MFMA_COEXEC_CYCLES") / (1024 * cyc2),
            100 * 4 * g(m2, "SQ_ACTIVE_INST_VALU") / (1024 * cyc2),
            100 * lds_act / (256 * cyc),
            100 * g(m1, "SQ_LDS_BANK_CONFLICT") / lds_act if lds_act else 0.0,
            100 * g(m2, "SQ_WAIT_INST_ANY") / g(m2, "SQ_WAVE_CYCLES") if g(m2, "SQ_WAVE_CYCLES") else 0.0,
            100 * g(m2, "SQ_WAIT_INST_LDS") / g(m2, "SQ_WAVE_CYCLES") if g(m2, "SQ_WAVE_CYCLES") else 0.0,
            512 * g(m1, "SQ_INSTS_VALU_MFMA_MOPS_BF16") / 1e12))
    open(os.path.join(args.out, "%s_utilisation.txt" % name), "w").write("\n".join(out) + "\n")
    shown = ["kernel_trace", "hbm_traffic", "utilisation"]
    # ---- optional: the vector-memory path (raw counter means per launch)
    if os.path.isdir(os.path.join(args.dir, "vmem")) and os.path.isdir(os.path.join(args.dir, "tc")):
        mm = {}
        for pname in MEMORY_PASSES:
            for ctr, rws in counter_rows(os.path.join(args.dir, pname)).items():
                if ctr != "GRBM_GUI_ACTIVE" or pname == "vmem":
                    mm[ctr] = mean_of(rws)
        cols = [c for c in mm if c != "GRBM_GUI_ACTIVE"]
        out = ["Vector-memory path per launch from rocprofv3 PMC counters over bench.py (raw counter values, mean per launch;"] + \
              ["SQ_* summed over the chip's SIMDs / wavefronts, TCP_* / TCC_* over their instances; cycles = GRBM_GUI_ACTIVE / 8)"] + head + \
              ["commands:", cmd("vmem"), cmd("tc"), ""]
        out.append("%-18s %-20s %12s " % ("call", "kernel", "cycles") + " ".join("%14s" % c.replace("SQ_", "").replace("_sum", "")[:14] for c in cols))
        for key in mm.get("GRBM_GUI_ACTIVE", {}):
            out.append("%-18s %-20s %12.0f " % (key[0], key[1], mm["GRBM_GUI_ACTIVE"][key] / 8.0) +
                       " ".join("%14.4g" % mm[c].get(key, float("nan")) for c in cols))
        open(os.path.join(args.out, "%s_memory_path.txt" % name), "w").write("\n".join(out) + "\n")
        shown.append("memory_path")
    for n in shown:
        print(open(os.path.join(args.out, "%s_%s.txt" % (name, n))).read())


def read_traffic(workload, profiles_dir=None):
    """(dict name -> bytes, source hash the table was measured on) from profiles/<workload>_hbm_traffic.txt,
    or ({}, None) when there is no such file."""
    path = os.path.join(profiles_dir or os.path.join(ROOT, "profiles"), "%s_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return {}, None
    table, sha = {}, None
    for line in open(path):
        p = line.split()
        if len(p) == 3 and p[0] == "traffic_bytes":
            table[p[1]] = int(p[2])
        elif len(p) == 2 and p[0] == "source_sha256":
            sha = p[1]
    return table, sha


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("collect", "tables"):
        p = sub.add_parser(name)
        p.add_argument("--workload", default="c3")
        p.add_argument("--dir", required=True, help="raw output of the passes (a scratch folder, not committed)")
        if name == "tables":
            p.add_argument("--out", default=os.path.join(ROOT, "profiles"))
            p.add_argument("--name", default=None, help="prefix of the files written (default: the workload; "
                                                        "bench.py --recompute-bwd reads <workload>_recompute)")
        else:
            p.add_argument("--memory-path", action="store_true", help="two more passes: vector-memory instruction and "
                                                                      "write-path counters")
            p.add_argument("--bench-args", default="", help="further bench.py flags for every pass, as one string "
                                                            "(e.g. --bench-args=--recompute-bwd)")
    args = ap.parse_args()
    (collect if args.cmd == "collect" else tables)(args)


if __name__ == "__main__":
    main()
