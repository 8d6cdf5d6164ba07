#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/.

Three runs of the same workload are expected in one directory (names are the -o prefixes):

  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload W --no-others --no-cpu-baseline
  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o fetch -- python3 bench.py --workload W --no-others --no-cpu-baseline --copy-calibration --steps 40
  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR -o write -- python3 bench.py --workload W --no-others --no-cpu-baseline --copy-calibration --steps 40

usage: python profile_summary.py DIR W
writes profiles/W_kernels.md and updates profiles/traffic.json (read back by bench.py for roofline.traffic).

usage: python profile_summary.py DIR W backward
DIR holds one run with the backward pass timed as well:
  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload W --no-others --no-cpu-baseline --backward --steps 30 --warmup 5
writes profiles/W_backward_kernels.md (durations of the backward pass's kernels only).

usage: python profile_summary.py DIR W counters [MODE]
DIR holds one run with eight SQ counters (MODE = pure, the default, or module):
  rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_LDS SQ_ACTIVE_INST_LDS SQ_LDS_BANK_CONFLICT --kernel-trace --output-format csv -d DIR -o sq -- python3 bench.py --workload W --mode MODE --no-others --no-cpu-baseline --steps 20 --warmup 5
writes profiles/W_sq_counters.md (profiles/W_module_sq_counters.md): per kernel the launch shape, registers,
LDS, the median of every counter per dispatch and the ratios used in the design notes.

HBM bytes: FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch; both are scaled by what the same
counter reads for the plain 1 GiB device-to-device copy that --copy-calibration runs (it moves exactly
1 GiB in and 1 GiB out), so a mis-scaled counter cancels out.
"""
import csv
import json
import os
import re
import statistics
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
GIB_KIB = float(1 << 20)


def short(name):
    name = re.sub(r"\(.*", "", name)
    return name.replace("void ", "").replace("aa::", "")


def stage_of(kernel):
    k = kernel.lower()
    if "fused" in k:
        return "small_fused"
    if "pool" in k:
        return "pool"
    if "aggregate" in k or "merge" in k:
        return "aggregate"
    if "broadcast" in k:
        return "broadcast"
    return None


def read_stats(path):
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            rows.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                         float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    return rows


def read_counter(path, counter):
    """kernel -> list of per-dispatch values of `counter`."""
    out = {}
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            out.setdefault(short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return out


def calibration(values_by_kernel):
    """Counter reading (KiB) of the 1 GiB copy: the largest dispatch among the runtime's copy kernels
    (the same kernel also serves the small host-to-device copies of the benchmark's set-up)."""
    best = None
    for k, v in values_by_kernel.items():
        if "copy" in k.lower():
            m = max(v)
            if best is None or m > best:
                best = m
    return best


BACKWARD_KERNELS = ("matmul_kernel", "mfma_matmul_kernel", "mfma_matmul_pair_kernel", "from_f32_x3_kernel",
                    "splitk_reduce_kernel", "softmax_rows", "softmax_grad_rows",
                    "value_extras_kernel", "dwc_param_grad_kernel", "bias_grad_kernel", "pool_grad_kernel", "to_f32_kernel",
                    "from_f32_kernel")


def backward_summary(d, wl):
    cmd = ("rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload %s "
           "--no-others --no-cpu-baseline --backward --steps 30 --warmup 5" % wl)
    lines = ["# rocprofv3 summary: backward pass, bench.py --workload %s --backward (one MI355X)" % wl, "",
             "command: `%s`" % cmd, "",
             "Kernels of `agent_attn_bwd` only (the run also times the forward pass; its kernels are in "
             "`%s_kernels.md`).  `us per backward` = calls x avg / number of backward calls." % wl, "",
             "| kernel | calls | avg us | us per backward |", "|---|---|---|---|"]
    rows = []
    with open(os.path.join(d, "stats_kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            name = r["Name"].replace("void ", "").replace("aa::(anonymous namespace)::", "").replace("aa::", "")
            name = re.sub(r"\(.*", "", name)
            if name.startswith(BACKWARD_KERNELS):
                rows.append((name, int(r["Calls"]), float(r["AverageNs"]) / 1e3))
    ncalls = min(c for n, c, a in rows if n.startswith("pool_grad_kernel") or n.startswith("from_f32_kernel")) if rows else 1
    pg = [c for n, c, a in rows if n.startswith("pool_grad_kernel")]
    ncalls = pg[0] if pg else ncalls
    total = 0.0
    for name, calls, avg in rows:
        per = calls * avg / ncalls
        total += per
        lines.append("| `%s` | %d | %.1f | %.1f |" % (name, calls, avg, per))
    lines += ["", "sum over the kernels: %.1f us per backward call (%d calls)" % (total, ncalls)]
    with open(os.path.join(ROOT, "profiles", "%s_backward_kernels.md" % wl), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


SQ_COUNTERS = ("SQ_BUSY_CU_CYCLES", "SQ_INSTS_VALU", "SQ_INSTS_MFMA", "SQ_ACTIVE_INST_VALU", "SQ_VALU_MFMA_BUSY_CYCLES",
               "SQ_INSTS_LDS", "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT")


def counters_summary(d, wl, mode):
    cmd = ("rocprofv3 --pmc %s --kernel-trace --output-format csv -d DIR -o sq -- python3 bench.py --workload %s "
           "--mode %s --no-others --no-cpu-baseline --steps 20 --warmup 5" % (" ".join(SQ_COUNTERS), wl, mode))
    per = {}
    with open(os.path.join(d, "sq_counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            k = short(r["Kernel_Name"])
            if not k.startswith(("small_", "pool_", "aggregate_", "merge_", "broadcast_", "large_", "bias_")):
                continue
            e = per.setdefault(k, {"c": {}, "dur": [], "shape": None})
            e["c"].setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
            e["dur"].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
            e["shape"] = (int(r["Grid_Size"]), int(r["Workgroup_Size"]), int(r["VGPR_Count"]), int(r["Accum_VGPR_Count"]),
                          int(r["LDS_Block_Size"]), int(r["Scratch_Size"]))
    lines = ["# SQ counters: bench.py --workload %s --mode %s (one MI355X)" % (wl, mode), "", "command: `%s`" % cmd, "",
             "Medians over the dispatches of each kernel; counter values are sums over the chip as rocprofv3 reports "
             "them.  Kernel durations under counter collection are longer than in the timing runs.", "",
             "| kernel | grid threads | block | VGPRs (+acc) | LDS B | scratch B | us under collection |",
             "|---|---|---|---|---|---|---|"]
    for k, e in sorted(per.items()):
        g, w, v, a, l, sc = e["shape"]
        lines.append("| `%s` | %d | %d | %d (+%d) | %d | %d | %.1f |" % (k, g, w, v, a, l, sc, statistics.median(e["dur"])))
    lines += ["", "| kernel | " + " | ".join(c.replace("SQ_", "") for c in SQ_COUNTERS) + " |",
              "|---|" + "---|" * len(SQ_COUNTERS)]
    med = {}
    for k, e in sorted(per.items()):
        med[k] = {c: statistics.median(e["c"].get(c, [0.0])) for c in SQ_COUNTERS}
        lines.append("| `%s` | " % k + " | ".join("%.3g" % med[k][c] for c in SQ_COUNTERS) + " |")
    lines += ["", "Ratios.  BUSY_CU_CYCLES and VALU_MFMA_BUSY_CYCLES count cycles (the latter reads 16 per "
              "16x16x32 MFMA); ACTIVE_INST_VALU reads about 1.1 per VALU instruction, i.e. it counts the four-cycle "
              "passes of a 64-lane instruction over the 16-lane SIMD, so VALU-active cycles = 4 x ACTIVE_INST_VALU.  "
              "Both pipes are given as a fraction of the SIMD cycles of the busy CUs (4 x BUSY_CU_CYCLES); the last "
              "column is bank-conflict cycles per LDS-active count.", "",
              "| kernel | VALU / MFMA insts | VALU active, fraction of SIMD cycles | MFMA busy, fraction of SIMD cycles | LDS conflict / LDS active |",
              "|---|---|---|---|---|"]

    def ratio(a, b):
        return "%.2f" % (a / b) if b > 0 else "-"

    for k, m in sorted(med.items()):
        busy4 = 4.0 * m["SQ_BUSY_CU_CYCLES"]
        lines.append("| `%s` | %s | %s | %s | %s |" % (k, ratio(m["SQ_INSTS_VALU"], m["SQ_INSTS_MFMA"]),
                                                      ratio(4.0 * m["SQ_ACTIVE_INST_VALU"], busy4),
                                                      ratio(m["SQ_VALU_MFMA_BUSY_CYCLES"], busy4),
                                                      ratio(m["SQ_LDS_BANK_CONFLICT"], m["SQ_ACTIVE_INST_LDS"])))
    name = "%s_sq_counters.md" % wl if mode == "pure" else "%s_%s_sq_counters.md" % (wl, mode)
    with open(os.path.join(ROOT, "profiles", name), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


def main():
    d, wl = sys.argv[1], sys.argv[2]
    if len(sys.argv) > 3 and sys.argv[3] == "backward":
        backward_summary(d, wl)
        return
    if len(sys.argv) > 3 and sys.argv[3] == "counters":
        counters_summary(d, wl, sys.argv[4] if len(sys.argv) > 4 else "pure")
        return
    lines = ["# rocprofv3 summary: bench.py --workload %s (one MI355X)" % wl, ""]
    stats_path = os.path.join(d, "stats_kernel_stats.csv")
    lines += ["## kernel durations (--kernel-trace --stats)", "",
              "command: `rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py "
              "--workload %s --no-others --no-cpu-baseline`" % wl, "",
              "`avg w/o max` leaves out the slowest dispatch (the first launch of a kernel pays for loading its "
              "code).", "",
              "| kernel | calls | avg us | avg w/o max | min us | max us | % of GPU time |", "|---|---|---|---|---|---|---|"]
    for name, calls, avg, mn, mx, pct in read_stats(stats_path):
        if name.startswith(("small_", "pool_", "aggregate_", "merge_", "broadcast_", "large_")):
            rest = (avg * calls - mx) / (calls - 1) if calls > 1 else avg
            lines.append("| `%s` | %d | %.2f | %.2f | %.2f | %.2f | %.2f |" % (name, calls, avg, rest, mn, mx, pct))
    traffic = {}
    fetch_p, write_p = os.path.join(d, "fetch_counter_collection.csv"), os.path.join(d, "write_counter_collection.csv")
    if os.path.exists(fetch_p) and os.path.exists(write_p):
        fetch, write = read_counter(fetch_p, "FETCH_SIZE"), read_counter(write_p, "WRITE_SIZE")
        cf, cw = calibration(fetch), calibration(write)
        lines += ["", "## HBM traffic per launch (--pmc FETCH_SIZE, --pmc WRITE_SIZE; separate runs)", "",
                  "commands: `rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o fetch -- python3 "
                  "bench.py --workload %s --no-others --no-cpu-baseline --copy-calibration --steps 40` and the same with "
                  "WRITE_SIZE / -o write." % wl, "",
                  "calibration: the 1 GiB device copy reads FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB "
                  "(expected 1048576 each) -> scale factors %.4f and %.4f." % (cf, cw, GIB_KIB / cf, GIB_KIB / cw), "",
                  "| kernel | fetch MB | write MB | total MB |", "|---|---|---|---|"]
        per_stage = {}
        for k in sorted(set(fetch) | set(write)):
            st = stage_of(k)
            if st is None or "copy" in k.lower():
                continue
            fb = statistics.median(fetch.get(k, [0.0])) * (GIB_KIB / cf) * 1024.0
            wb = statistics.median(write.get(k, [0.0])) * (GIB_KIB / cw) * 1024.0
            lines.append("| `%s` | %.2f | %.2f | %.2f |" % (k, fb / 1e6, wb / 1e6, (fb + wb) / 1e6))
            e = per_stage.setdefault(st, {"fetch": 0.0, "write": 0.0})
            e["fetch"] += fb
            e["write"] += wb
        for st, e in per_stage.items():
            traffic[st] = {"hbm_bytes_per_launch": e["fetch"] + e["write"], "fetch_bytes": e["fetch"],
                           "write_bytes": e["write"]}
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", "%s_kernels.md" % wl), "w") as f:
        f.write("\n".join(lines) + "\n")
    if traffic:
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        table = {}
        if os.path.exists(tpath):
            with open(tpath) as f:
                table = json.load(f)
        table[wl] = traffic
        with open(tpath, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
    print("\n".join(lines))


if __name__ == "__main__":
    main()
