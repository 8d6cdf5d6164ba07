#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/.

usage: python profile_summary.py DIR W
DIR holds, for workload W,
  stats_kernel_stats.csv   from  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload W --no-others --no-cpu-baseline --no-traffic
  bench_profiled.json      the JSON line that run printed (kernel durations from HIP events, taken under the profiler)
  bench.json               the JSON line of a plain  python3 bench.py --workload W --no-others --no-cpu-baseline
                           (kernel durations from HIP events, and HBM bytes per launch from the two rocprofv3 --pmc
                           FETCH_SIZE / WRITE_SIZE child runs that bench.py makes itself, scaled by a copy of known size)
writes profiles/W_kernels.md: per kernel the profiler's average duration next to the benchmark's own, the measured
HBM bytes per launch next to the algorithmic ones, and the roofline entry of the dominant kernel.

usage: python profile_summary.py DIR W backward [MODE]
DIR holds one run with the backward pass timed as well (MODE = pure, the default, or module):
  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload W --mode MODE --no-others --no-cpu-baseline --no-traffic --backward --steps 30 --warmup 5
writes profiles/W_backward_kernels.md (profiles/W_module_backward_kernels.md): durations of the backward pass's
kernels only.

usage: python profile_summary.py DIR W counters [MODE]
DIR holds one run with eight SQ counters (MODE = pure, the default, module, or backward = pure with --backward
added to the bench.py command: then only the backward pass's kernels are listed):
  rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_LDS SQ_ACTIVE_INST_LDS SQ_LDS_BANK_CONFLICT --kernel-trace --output-format csv -d DIR -o sq -- python3 bench.py --workload W --mode MODE --no-others --no-cpu-baseline --no-traffic --steps 20 --warmup 5
writes profiles/W_sq_counters.md (profiles/W_module_sq_counters.md): per kernel the launch shape, registers,
LDS, the median of every counter per dispatch and the ratios used in the design notes.
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
    name = re.sub(r"\(.*", "", name.replace("(anonymous namespace)::", ""))
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
                    "value_extras_kernel", "dwc_param_partial_kernel", "dwc_param_sum_kernel", "batch_sum_kernel",
                    "bias_grad_kernel", "bias_grad_row_kernel", "pool_grad_kernel", "to_f32_kernel",
                    "from_f32_kernel", "fused_token_kernel", "fused_agent_kernel", "fused_merge_kernel",
                    "fused_reduce_bc_kernel", "fused_reduce_agg_kernel")


def backward_summary(d, wl, mode="pure"):
    cmd = ("rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload %s "
           "--mode %s --no-others --no-cpu-baseline --no-traffic --backward --steps 30 --warmup 5" % (wl, mode))
    lines = ["# rocprofv3 summary: backward pass, bench.py --workload %s --mode %s --backward (one MI355X)" % (wl, mode), "",
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
    # kernels that run once per backward call
    once = [c for n, c, a in rows if n.startswith(("fused_merge_kernel", "pool_grad_kernel", "from_f32_x3_kernel"))]
    ncalls = min(once) if once else 1
    total = 0.0
    for name, calls, avg in rows:
        per = calls * avg / ncalls
        total += per
        lines.append("| `%s` | %d | %.1f | %.1f |" % (name, calls, avg, per))
    lines += ["", "sum over the kernels: %.1f us per backward call (%d calls)" % (total, ncalls)]
    name = "%s_backward_kernels.md" % wl if mode == "pure" else "%s_%s_backward_kernels.md" % (wl, mode)
    with open(os.path.join(ROOT, "profiles", name), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


SQ_COUNTERS = ("SQ_BUSY_CU_CYCLES", "SQ_INSTS_VALU", "SQ_INSTS_MFMA", "SQ_ACTIVE_INST_VALU", "SQ_VALU_MFMA_BUSY_CYCLES",
               "SQ_INSTS_LDS", "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT")


BACKWARD_FUSED = ("fused_token_kernel", "fused_agent_kernel", "fused_merge_kernel", "fused_reduce_")


def counters_summary(d, wl, mode):
    bench_mode = "pure --backward" if mode == "backward" else mode
    cmd = ("rocprofv3 --pmc %s --kernel-trace --output-format csv -d DIR -o sq -- python3 bench.py --workload %s "
           "--mode %s --no-others --no-cpu-baseline --no-traffic --steps 20 --warmup 5" % (" ".join(SQ_COUNTERS), wl, bench_mode))
    per = {}
    with open(os.path.join(d, "sq_counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            k = short(r["Kernel_Name"])
            if not k.startswith(("small_", "pool_", "aggregate_", "merge_", "broadcast_", "large_", "bias_", "fused_",
                                 "(anonymous namespace)::fused_")):
                continue
            if (mode == "backward") != k.startswith(BACKWARD_FUSED):      # the backward's kernels, or all the others
                continue
            e = per.setdefault(k, {"c": {}, "dur": [], "shape": None})
            e["c"].setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
            e["dur"].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
            e["shape"] = (int(r["Grid_Size"]), int(r["Workgroup_Size"]), int(r["VGPR_Count"]), int(r["Accum_VGPR_Count"]),
                          int(r["LDS_Block_Size"]), int(r["Scratch_Size"]))
    lines = ["# SQ counters: bench.py --workload %s --mode %s (one MI355X)" % (wl, bench_mode), "", "command: `%s`" % cmd, "",
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
        backward_summary(d, wl, sys.argv[4] if len(sys.argv) > 4 else "pure")
        return
    if len(sys.argv) > 3 and sys.argv[3] == "counters":
        counters_summary(d, wl, sys.argv[4] if len(sys.argv) > 4 else "pure")
        return
    kernels_summary(d, wl)


def launcher_of(kernel):
    """Launcher name that bench.py reports for a profiler kernel name."""
    k = re.sub(r"<.*", "", kernel.replace("(anonymous namespace)::", "")).split("::")[-1]
    table = [("small_fused", "small_fused"), ("fused_f32", "fused_f32"), ("small_pool", "small_pool"),
             ("small_aggregate", "small_aggregate"), ("small_merge", "small_merge"), ("small_broadcast", "small_broadcast"),
             ("large_agents", "large_agents"), ("large_aggregate3", "large_aggregate2"), ("large_merge3", "large_merge2"),
             ("large_broadcast3", "large_broadcast2"), ("restride", "restride"), ("pool_generic", "pool_generic"),
             ("pool_vec", "pool_generic"), ("aggregate_generic", "aggregate_generic"), ("merge_generic", "merge_generic"),
             ("broadcast_generic", "broadcast_generic")]
    for prefix, name in table:
        if k.startswith(prefix):
            return name
    return None


def kernels_summary(d, wl):
    with open(os.path.join(d, "bench.json")) as f:
        plain = json.loads(f.read().strip().splitlines()[-1])
    with open(os.path.join(d, "bench_profiled.json")) as f:
        prof = json.loads(f.read().strip().splitlines()[-1])
    stats = {}
    for name, calls, avg, mn, mx, pct in read_stats(os.path.join(d, "stats_kernel_stats.csv")):
        ln = launcher_of(name)
        if ln:
            rest = (avg * calls - mx) / (calls - 1) if calls > 1 else avg
            stats.setdefault(ln, []).append((name, calls, avg, rest, mn, mx))
    lines = ["# rocprofv3 summary: bench.py --workload %s (one MI355X)" % wl, "",
             "commands:", "",
             "    rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o stats -- python3 bench.py --workload %s --no-others --no-cpu-baseline --no-traffic" % wl,
             "    python3 bench.py --workload %s --no-others --no-cpu-baseline      (HIP-event durations without the profiler; HBM bytes from its own two rocprofv3 --pmc runs)" % wl, "",
             "workload: %s" % json.dumps(plain["config"]), "",
             "step (all kernels of one forward pass, cold inputs): %.2f us plain, %.2f us under the profiler" % (
                 plain["ms_per_step"] * 1e3, prof["ms_per_step"] * 1e3), "",
             "`profiler avg` is rocprofv3's average over all dispatches, `w/o max` leaves out the slowest one (the first launch of "
             "a kernel pays for loading its code); `events` is what bench.py measures itself with HIP events recorded between "
             "the launches (it includes the gap to the next launch), plain and under the profiler.", "",
             "| kernel (launcher) | calls | profiler avg us | w/o max | min | max | events us (plain) | events us (profiled) | HBM MB / launch (measured) |",
             "|---|---|---|---|---|---|---|---|---|"]
    pk = {k["name"].split("_dp")[0]: k for k in prof["kernels"]}
    for k in plain["kernels"]:
        ln = k["name"].split("_dp")[0]
        rows = stats.get(ln, [])
        hb = "%.2f" % (k["hbm_bytes"] / 1e6) if k.get("hbm_bytes") else "-"
        ev2 = "%.2f" % pk[ln]["avg_us"] if ln in pk else "-"
        if not rows:
            lines.append("| `%s` | - | - | - | - | - | %.2f | %s | %s |" % (k["name"], k["avg_us"], ev2, hb))
        for name, calls, avg, rest, mn, mx in rows:
            lines.append("| `%s` (`%s`) | %d | %.2f | %.2f | %.2f | %.2f | %.2f | %s | %s |" % (
                short(name)[:60], k["name"], calls, avg, rest, mn, mx, k["avg_us"], ev2, hb))
    r = plain["roofline"]
    lines += ["", "roofline of the dominant kernel (bench.py): `%s`" % json.dumps(r), "",
              "traffic source: %s" % plain.get("traffic_source"), ""]
    if "algorithmic_path_bytes" in plain or "path_hbm_bytes_measured" in plain:
        lines.append("whole path: algorithmic bytes %s, measured HBM bytes %s" % (
            plain.get("algorithmic_path_bytes"), plain.get("path_hbm_bytes_measured")))
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", "%s_kernels.md" % wl), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
