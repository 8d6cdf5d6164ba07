"""Checks on the compiler's output for the kernels that issue LDS reads behind the compiler's back.

The large-agent kernels place some operand reads by hand: a `ds_read` inside an asm statement, and later an
`s_waitcnt lgkmcnt(n)` asm statement that ties the registers.  Between the two the compiler believes the registers
already hold their values, so nothing it emits may read or write them before the wait that covers them (a copy
would take stale data, a reuse would be overwritten when the read arrives).  This test compiles the three
large-agent units to gfx950 assembly with the build's flags and scans every kernel in emission order: LDS reads
of a wave complete in order, so after a hand-written `lgkmcnt(n)` only the youngest n hand-issued reads are still
in flight."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import __graft_entry__ as entry      # noqa: E402


def _regs(tok):
    tok = tok.strip()
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def scan_in_flight(text):
    """Returns (number of hand-issued reads seen, list of offending lines)."""
    in_asm, flight, issued, bad, kernel = False, [], 0, [], ""
    for ln, line in enumerate(text.split("\n"), 1):
        t = line.strip()
        if re.match(r"^_Z\w+:", line):
            kernel, flight = line.split(":")[0], []
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t[0] in ";.":
            continue
        op = t.split()[0]
        ops = t.split(None, 1)[1].split(",") if " " in t else []
        wait = re.search(r"lgkmcnt\((\d+)\)", t) if op == "s_waitcnt" else None
        if in_asm:
            if op.startswith("ds_read"):
                flight.append((_regs(ops[0]), ln))
                issued += 1
            elif wait:
                n = int(wait.group(1))
                flight = flight[len(flight) - n:] if n else []
            continue
        if wait and int(wait.group(1)) == 0:      # the compiler's own full wait covers them as well
            flight = []
            continue
        if op == "s_endpgm":
            flight = []
            continue
        used = set()
        for o in ops:
            used |= _regs(o.split()[0] if o.strip() else "")
        for rs, at in flight:
            if used & rs:
                bad.append("%s line %d: '%s' touches v%s, in flight since line %d" % (kernel[:60], ln, t[:60],
                                                                                   sorted(used & rs)[:4], at))
                break
    return issued, bad


def test_scanner_sees_a_planted_touch():
    text = ("_Zfoo:\n\t;;#ASMSTART\n\tds_read_b128 v[4:7], v1 offset:0\n\t;;#ASMEND\n\tv_mov_b32_e32 v9, v5\n"
            "\t;;#ASMSTART\n\ts_waitcnt lgkmcnt(0)\n\t;;#ASMEND\n\tv_mov_b32_e32 v9, v5\n")
    issued, bad = scan_in_flight(text)
    assert issued == 1 and len(bad) == 1 and "line 5" in bad[0]


def test_no_instruction_touches_a_register_with_a_hand_issued_read_in_flight(tmp_path):
    units = ["large_agent_dp32.hip", "large_agent_dp64.hip", "large_agent_dp128.hip"]
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-Wall")] + ["-fno-honor-nans", "-S", "--cuda-device-only"]
    procs = []
    for u in units:
        out = str(tmp_path / (u + ".s"))
        procs.append((u, out, subprocess.Popen(["hipcc"] + flags + [os.path.join(entry.CSRC, u), "-o", out],
                                               stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for u, out, p in procs:
        log, _ = p.communicate()
        assert p.returncode == 0, log
        issued, bad = scan_in_flight(open(out).read())
        assert issued > 100, "%s: the hand-issued reads were not found (%d)" % (u, issued)
        assert not bad, "\n".join(bad[:10])


def test_backward_product_kernels_keep_their_accumulators_in_ordinary_registers(tmp_path):
    """The MFMA kernels of the backward pass ask for two blocks per CU, i.e. at most 256 registers per lane: then
    the compiler has no reason to place MFMA accumulators in the accumulator file, and every copy in or out of it
    (`v_accvgpr_read` / `_write`) would be a vector instruction spent on nothing.  The recomputing kernels are
    bound by their vector arithmetic, so the copies cost a tenth of their time when they were there."""
    units = ["backward_fused_kernels.hip", "backward_kernels.hip"]
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-Wall")] + ["-S", "--cuda-device-only"]
    procs = []
    for u in units:
        out = str(tmp_path / (u + ".s"))
        procs.append((u, out, subprocess.Popen(["hipcc"] + flags + [os.path.join(entry.CSRC, u), "-o", out],
                                               stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for u, out, p in procs:
        log, _ = p.communicate()
        assert p.returncode == 0, log
        text = open(out).read()
        assert text.count("v_mfma_f32_16x16x32") > 50, u
        # per kernel; the aggregation's token kernel at head width 128 needs more than 256 registers and is left
        # at one block per CU (template arguments <E, 128, kAgg = 2, 2>)
        kernel, counts = "", {}
        for line in text.split("\n"):
            if re.match(r"^_Z\w+:", line):
                kernel = line.split(":")[0]
            elif "v_accvgpr" in line:
                counts[kernel] = counts.get(kernel, 0) + 1
        counts = {k: c for k, c in counts.items() if not ("fused_token_kernel" in k and "ELi128ELi2ELi2E" in k)}
        assert not counts, "%s: accumulator-file copies in %s" % (u, sorted(counts.items())[:4])
