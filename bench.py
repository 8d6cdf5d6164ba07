#!/usr/bin/env python3
"""Benchmark of the agent-attention forward pass on one MI355X.

A step is one pass of the whole hot path (agents, aggregation + merge, broadcast) over one batch of
seeded synthetic inputs that already sit in HBM.  Steps rotate over a ring of input/output sets larger
than the 256 MB Infinity Cache so that every step reads its inputs from HBM ("cold").  Prints ONE JSON
line.  The headline workload is the largest single-GPU configuration (`highres`); every other workload
gets the same measurements under "workloads".

Per workload:
  * step time over K back-to-back calls of agent_attn_fwd (HIP events on the launch stream);
  * the duration of every kernel the call launches (agent_attn_fwd_timed: events between the launches);
  * roofline of the dominant kernel: algorithmic bytes (HBM-bound shapes, n <= 256) or FLOPs (n = 1024)
    of its stage per launch / its average duration, against 8 TB/s or the dense bf16/fp16 MFMA peak;
  * HBM traffic per launch of every kernel from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this
    script in a child mode, made before this process touches the GPU, scaled by what the same counters
    read for a copy of known size (null when rocprofv3 is not usable);
  * the fp64 CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload highres] [--mode pure|module]
"""
import argparse
import csv
import json
import os
import shutil
import statistics
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, GB/s
MFMA_PEAK_TFLOPS = 2516.6      # dense bf16 / fp16 MFMA: 256 CUs x 2.4 GHz x 4096 FLOP/clk/CU
VALU_F32_PEAK_TFLOPS = 157.3   # fp32 vector arithmetic, published figure, TFLOP/s
ELEM = {"f32": 4, "f16": 2, "bf16": 2}
DT = {"f32": 0, "f16": 1, "bf16": 2}
ORDER = ("highres", "sd_latent", "swin_t_s1", "deit_t", "tiny")
CALIBRATION_BYTES = 1 << 30


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="highres")
    ap.add_argument("--mode", default="pure", choices=["pure", "module"])
    ap.add_argument("--backward", action="store_true",
                    help="also time agent_attn_bwd on the workload and add a \"backward\" object to the line")
    ap.add_argument("--ring-bytes", type=float, default=1.25e9, help="total footprint of the rotating input sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-traffic", action="store_true", help="skip the rocprofv3 counter runs (roofline.traffic = null)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the steps from a captured HIP graph (one graph = one pass over the ring)")
    ap.add_argument("--traffic-pass", metavar="JSON",
                    help="child mode of the counter runs: a copy of known size, then a few cold steps of every workload "
                         "in --workloads; writes what it launched to JSON")
    ap.add_argument("--workloads", default="", help="comma-separated list for --traffic-pass")
    return ap.parse_args()


def stage_bytes(wl):
    """Algorithmic HBM bytes per launch of each stage and of the whole path (all units)."""
    s, u = ELEM[wl.dtype], wl.units
    big, small = u * wl.N * wl.d * s, u * wl.n * wl.d
    return {
        "pool": big + small * s,                       # read Q, write A
        "aggregate": 2 * big + small * s + small * 4,  # read K, V, A; write V_A
        "broadcast": 2 * big + small * s + small * 4,  # read Q, A, V_A; write O
        "merge": 2 * small * 4,
        "path": 4 * big,                               # read Q, K, V once, write O once
    }


def stage_flops(wl):
    f = 4.0 * wl.N * wl.n * wl.d * wl.units
    return {"pool": 0.0, "merge": 0.0, "aggregate": f, "broadcast": f, "path": 2 * f}


def stage_of(kernel_name):
    k = kernel_name.lower()
    if "fused" in k:
        return "path"
    if "pool" in k or "agents" in k:
        return "pool"
    if "merge" in k:
        return "merge"
    if "aggregate" in k:
        return "aggregate"
    if "broadcast" in k:
        return "broadcast"
    return None


class Ring:
    """R independent copies of (Q, K, V, out, workspace) on the device."""

    def __init__(self, wl, binding, ring_bytes, module, prepared=False):
        import numpy as np
        import torch
        from paper_2312_08874_amd import inputs
        self.wl, self.binding = wl, binding
        t = inputs.make_qkv(wl)
        shape = (wl.batch, wl.heads, wl.N, wl.d)

        def dev(a):
            if wl.dtype == "bf16":
                return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).reshape(shape).cuda()
            return torch.from_numpy(a).reshape(shape).cuda()

        base = {k: dev(v) for k, v in t.items()}
        self.host = t
        self.params = None
        self.host_params = None
        if module:
            self.host_params = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, index=wl.index)
            self.params = {k: torch.from_numpy(v).cuda() for k, v in self.host_params.items()}
            if prepared:      # agent-bias tables built once, outside the timed calls (fixed parameters: inference)
                tables = binding.agent_attn_bias_tables(self.params, heads=wl.heads, N=wl.N, n=wl.n, d=wl.d,
                                                        dtype=base["Q"].dtype, grid=wl.grid)
                if tables is not None:
                    self.params["bias_tables"] = tables
        desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, DT[wl.dtype], wl.grid, wl.agent_grid)
        ws_bytes = max(256, binding.workspace_bytes(desc, binding.make_params(self.params)))
        per_set = 4 * base["Q"].numel() * base["Q"].element_size() + ws_bytes
        self.R = max(2, min(256, int(ring_bytes // per_set) + 1))
        self.sets = []
        for _ in range(self.R):
            s = {k: v.clone() for k, v in base.items()}
            s["out"] = torch.empty_like(base["Q"])
            s["ws"] = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
            self.sets.append(s)
        b, p = binding, self.params
        self.fwd = [b.prepare_fwd(s["Q"], s["K"], s["V"], grid=wl.grid, agent_grid=wl.agent_grid, params=p,
                                  out=s["out"], workspace=s["ws"]) for s in self.sets]

    def forward(self, i):
        self.fwd[i % self.R]()

    def forward_timed(self, i):
        s = self.sets[i % self.R]
        return self.binding.agent_attn_fwd_timed(s["Q"], s["K"], s["V"], grid=self.wl.grid, agent_grid=self.wl.agent_grid,
                                                 params=self.params, out=s["out"], workspace=s["ws"])


def timed(fn, steps, warmup):
    """Average milliseconds per call over `steps` back-to-back calls, HIP events on the launch stream."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def timed_graph(ring, steps, warmup):
    """Same measurement with the launches replayed from a HIP graph that holds one pass over the ring."""
    import torch
    for i in range(max(warmup, ring.R)):
        ring.forward(i)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        calls = [ring.binding.prepare_fwd(s["Q"], s["K"], s["V"], grid=ring.wl.grid, agent_grid=ring.wl.agent_grid,
                                          params=ring.params, out=s["out"], workspace=s["ws"], stream=side)
                 for s in ring.sets]
        for c in calls:
            c()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for c in calls:
                c()
    torch.cuda.synchronize()
    reps = max(1, steps // ring.R)
    graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (reps * ring.R)


def kernel_times(ring, steps, warmup):
    """[(launcher name, average microseconds)] of the kernels one forward call launches, cold ring."""
    for i in range(max(2, warmup // 4)):
        ring.forward_timed(i)
    acc = None
    for i in range(steps):
        t = ring.forward_timed(warmup + i)
        if acc is None:
            acc = [[name, 0.0] for name, _ in t]
        for slot, (_, ms) in zip(acc, t):
            slot[1] += ms
    return [(name, total / steps * 1e3) for name, total in acc]


def roofline_for(wl, kernels, traffic):
    """Roofline entry of the dominant kernel (longest average launch among the kernels of a step)."""
    idx = max(range(len(kernels)), key=lambda i: kernels[i][1])
    name, us = kernels[idx]
    stage = stage_of(name) or "path"
    t = None
    if traffic and idx < len(traffic) and traffic[idx] is not None:
        t = traffic[idx]["hbm_bytes"]
    if wl.n >= 1024:
        ach = stage_flops(wl)[stage] / (us * 1e-6) / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_PEAK_TFLOPS, "traffic": t, "avg_launch_us": us,
                "algorithmic_flops_per_launch": stage_flops(wl)[stage]}
    ach = stage_bytes(wl)[stage] / (us * 1e-6) / 1e9
    return {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": t, "avg_launch_us": us,
            "algorithmic_bytes_per_launch": stage_bytes(wl)[stage]}


def step_time(wl, binding, ring_bytes, steps, warmup, module, prepared=False):
    """Milliseconds per forward pass alone, for the hot and module-mode variants."""
    import torch
    ring = Ring(wl, binding, ring_bytes, module, prepared)
    ms = timed(ring.forward, steps, warmup)
    del ring
    torch.cuda.empty_cache()
    return ms


def measured_copy_gbs():
    """What a plain device-to-device copy of 1 GiB reaches on this GPU (bytes read + bytes written per
    second): the practical ceiling next to the 8 TB/s peak that the roofline fraction is quoted against."""
    import torch
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ms = timed(lambda i: dst.copy_(src), 10, 3)
    del src, dst
    torch.cuda.empty_cache()
    return 2.0 * (1 << 30) / (ms * 1e-3) / 1e9


def single_call_latency_us(wl, binding):
    """Host-visible latency of one isolated forward call: enqueue + wait, median of 30 (launch-bound
    problems such as the fp32 parity configuration are priced by this, not by a roofline)."""
    import torch
    ring = Ring(wl, binding, 1.0, False)
    for i in range(5):
        ring.forward(i)
    torch.cuda.synchronize()
    samples = []
    for i in range(30):
        t0 = time.perf_counter()
        ring.forward(i)
        torch.cuda.synchronize()
        samples.append((time.perf_counter() - t0) * 1e6)
    del ring
    torch.cuda.empty_cache()
    return statistics.median(samples)


def module_with_projections_us(wl, binding, steps=30, warmup=5):
    """The module with its projections (agent_attn_module_fwd: q | k | v GEMM, agent attention, output GEMM) on the
    workload's shape, x [B, N, heads * d] resident in HBM, same inputs every call (hot); microseconds per call."""
    import torch
    C = wl.heads * wl.d
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[wl.dtype]
    g = torch.Generator(device="cuda").manual_seed(20231214)
    x = torch.randn((wl.batch, wl.N, C), generator=g, device="cuda", dtype=torch.float32).to(tdt)
    w_qkv = (torch.randn((3 * C, C), generator=g, device="cuda", dtype=torch.float32) * C ** -0.5).to(tdt)
    w_out = (torch.randn((C, C), generator=g, device="cuda", dtype=torch.float32) * C ** -0.5).to(tdt)
    y = torch.empty_like(x)
    desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, {"f32": 0, "f16": 1, "bf16": 2}[wl.dtype], wl.grid,
                             wl.agent_grid)
    import ctypes
    need = int(binding.lib().agent_attn_module_workspace_bytes(ctypes.byref(desc), None))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    call = lambda: binding.agent_attn_module_fwd(x, w_qkv, None, w_out, None, heads=wl.heads, grid=wl.grid,
                                                 agent_grid=wl.agent_grid, out=y, workspace=ws)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    del x, w_qkv, w_out, y, ws
    torch.cuda.empty_cache()
    return e0.elapsed_time(e1) / steps * 1e3


def measure(wl, binding, args, steps, warmup, module, traffic):
    ring = Ring(wl, binding, args.ring_bytes, module)
    ms = timed_graph(ring, steps, warmup) if args.graph else timed(ring.forward, steps, warmup)
    kernels = kernel_times(ring, max(10, min(steps, 60)), warmup)
    tokens = wl.batch * wl.N
    desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, DT[wl.dtype], wl.grid, wl.agent_grid)
    res = {
        "ms_per_step": ms,
        "tokens_per_s": tokens / (ms * 1e-3),
        "tflops": stage_flops(wl)["path"] / (ms * 1e-3) / 1e12,
        "path_gbs": stage_bytes(wl)["path"] / (ms * 1e-3) / 1e9,
        "dtype": wl.dtype,
        "kernels": [{"name": n, "avg_us": us,
                     "hbm_bytes": (traffic[i]["hbm_bytes"] if traffic and i < len(traffic) and traffic[i] else None)}
                    for i, (n, us) in enumerate(kernels)],
        "roofline": roofline_for(wl, kernels, traffic),
        "plan": binding.plan_str(desc),
        "ring_sets": ring.R,
        "algorithmic_path_bytes": stage_bytes(wl)["path"],
    }
    if traffic and all(t is not None for t in traffic):
        res["path_hbm_bytes_measured"] = sum(t["hbm_bytes"] for t in traffic)
    res["path_roofline_frac"] = (res["tflops"] / MFMA_PEAK_TFLOPS) if wl.n >= 1024 else (res["path_gbs"] / HBM_PEAK_GBS)
    return res, ring


def measure_backward(wl, binding, ring, steps, warmup):
    """agent_attn_bwd on the first input set (same buffers every call).  20*N*n*d FLOPs per unit in ten matrix
    products (the score tiles a 16-bit pure-mode problem recomputes are not counted): on MFMA for fp16 / bf16
    (priced against the dense MFMA peak), as fp32 vector FMAs for fp32 (priced against the fp32 vector peak)."""
    import ctypes
    import torch
    s = ring.sets[0]
    dO = torch.randn(s["Q"].shape, device="cuda", dtype=torch.float32).to(s["Q"].dtype)
    desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, DT[wl.dtype], wl.grid, wl.agent_grid)
    need = int(binding.lib().agent_attn_bwd_workspace_bytes(ctypes.byref(desc), binding._pp(binding.make_params(ring.params))))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def call(i):
        binding.agent_attn_bwd(s["Q"], s["K"], s["V"], dO, grid=wl.grid, agent_grid=wl.agent_grid, params=ring.params,
                               workspace=ws)
    ms = timed(call, steps, warmup)
    fused = wl.dtype != "f32" and ring.params is None and wl.d % 8 == 0 and wl.d <= 128
    flops = 20.0 * wl.N * wl.n * wl.d * wl.units
    tf = flops / (ms * 1e-3) / 1e12
    peak = VALU_F32_PEAK_TFLOPS if wl.dtype == "f32" else MFMA_PEAK_TFLOPS
    return {"ms_per_step": ms, "tokens_per_s": wl.batch * wl.N / (ms * 1e-3), "tflops": tf,
            "workspace_bytes": need, "cache": "hot (one input set)",
            "kernels": ("token kernels (dQ, dK, dV) + agent kernels (V_A, dV_A, dA) that recompute their score tiles, "
                        "no attention matrix in memory") if fused else
                       ("reference-quality: 10 batched matrix products + row softmax / gradient kernels, attention "
                        "matrices materialised in the workspace"),
            "roofline": {"kernel": "fused_token_kernel + fused_agent_kernel" if fused else
                         ("matmul_kernel" if wl.dtype == "f32" else "mfma_matmul_kernel"),
                         "bound": "alu" if wl.dtype == "f32" else "mfma", "achieved": tf, "peak": peak,
                         "unit": "TFLOP/s", "frac": tf / peak, "traffic": None}}


def oracle_dense_biases(oracle, params, heads, n, grid):
    """B1 [heads,n,N], B2 [heads,N,n] (float64) from the bias components via the oracle's own helper."""
    import numpy as np
    h, w = grid
    B1 = np.stack([oracle.bias1_dense(params["b1_col"][hd], params["b1_row"][hd], params["b1_blk"][hd], n, h, w)
                   for hd in range(heads)])
    B2 = np.stack([oracle.bias2_dense(params["b2_col"][hd], params["b2_row"][hd], params["b2_blk"][hd], n, h, w)
                   for hd in range(heads)])
    return B1, B2


def cpu_baseline(wl, ring):
    """The fp64 oracle, as it stands, on the host cores: a bounded sample of the same workload."""
    from oracle import agent_attn_oracle as oracle
    from paper_2312_08874_amd import inputs
    flops_unit = 8.0 * wl.N * wl.n * wl.d
    units = int(max(1, min(wl.units, 1.2e10 // flops_unit)))
    t = {k: v[:units] for k, v in ring.host.items()}
    q, k, v = (inputs.to_float64(t[x], wl.dtype) for x in ("Q", "K", "V"))
    kw = {}
    if ring.host_params:
        B1, B2 = oracle_dense_biases(oracle, ring.host_params, wl.heads, wl.n, wl.grid)
        kw = dict(B1=B1, B2=B2, dwc_w=ring.host_params["dwc_w"], dwc_b=ring.host_params["dwc_b"])
    heads = wl.heads if units % wl.heads == 0 else 1
    if heads == 1 and kw:
        kw = {kk: vv[:1] for kk, vv in kw.items()}
    small = min(units, 1)
    oracle.agent_attn_fwd(q[:small, :64], k[:small, :64], v[:small, :64], heads=1, A=q[:small, :4])      # warm the library
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < 1.5 and reps < 200:          # about 1.5 s of wall time on all host cores, at least one repetition
        oracle.agent_attn_fwd(q, k, v, heads=heads, grid=wl.grid, agent_grid=wl.agent_grid, **kw)
        reps += 1
        dt = time.perf_counter() - t0
    tokens = reps * units * wl.N / wl.heads
    return {"value": tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d (batch*head) units of workload %s, fp64, %d repetition(s), %.2f s wall"
                      % (units, wl.units, wl.name, reps, dt)}


# ---------------------------------------------------------------------------------------------------
# HBM traffic per kernel launch: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE around a child run of this script
# ---------------------------------------------------------------------------------------------------
def traffic_pass(args):
    """Child mode (run under rocprofv3): a device copy of CALIBRATION_BYTES, then cold forward steps of
    each workload in order.  Writes the launch bookkeeping the parent needs to JSON."""
    import torch
    from paper_2312_08874_amd import binding, inputs
    binding.lib()
    torch.cuda.set_device(0)
    src = torch.empty(CALIBRATION_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1, out=dst)      # an ordinary kernel that reads and writes exactly CALIBRATION_BYTES
    torch.cuda.synchronize()
    del src, dst
    torch.cuda.empty_cache()
    book = []
    for name in [w for w in args.workloads.split(",") if w]:
        wl = inputs.WORKLOADS[name]
        ring = Ring(wl, binding, min(args.ring_bytes, 6.0e8), args.mode == "module")
        per_step = len(ring.forward_timed(0))
        steps = 12
        for i in range(steps):
            ring.forward(1 + i)
        torch.cuda.synchronize()
        book.append({"workload": name, "first_call_kernels": per_step, "steps": steps, "kernels_per_step": per_step})
        del ring
        torch.cuda.empty_cache()
    with open(args.traffic_pass, "w") as f:
        json.dump(book, f)


def read_counter_rows(path, counter):
    """[(kernel name, value)] in dispatch order."""
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows.append((int(r["Dispatch_Id"]), r["Kernel_Name"], float(r["Counter_Value"])))
    rows.sort()
    return [(k, v) for _, k, v in rows]


def measure_traffic(workloads, mode, ring_bytes):
    """{workload: [per kernel of a step: {"hbm_bytes", "fetch_bytes", "write_bytes"}]} or {} when rocprofv3
    cannot be used.  Must run before this process initialises the GPU (it starts child processes)."""
    exe = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(exe):
        return {}, "rocprofv3 not found"
    out = {}
    tmp = tempfile.mkdtemp(prefix="aa_traffic_", dir="/tmp")
    try:
        per_counter = {}
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            book_path = os.path.join(tmp, "book_%s.json" % counter)
            cmd = [exe, "--pmc", counter, "--kernel-trace", "--output-format", "csv", "-d", os.path.join(tmp, counter),
                   "-o", "t", "--", sys.executable, os.path.join(ROOT, "bench.py"), "--traffic-pass", book_path,
                   "--workloads", ",".join(workloads), "--mode", mode, "--ring-bytes", str(ring_bytes)]
            env = dict(os.environ, TMPDIR="/tmp")
            r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=240)
            csvs = []
            for base, _, files in os.walk(os.path.join(tmp, counter)):
                csvs += [os.path.join(base, f) for f in files if f.endswith("counter_collection.csv")]
            if r.returncode != 0 or not csvs or not os.path.exists(book_path):
                return {}, "rocprofv3 --pmc %s failed (rc %d)" % (counter, r.returncode)
            with open(book_path) as f:
                book = json.load(f)
            rows = read_counter_rows(csvs[0], counter)
            lib_rows = [(k, v) for k, v in rows if "aa::" in k]
            other = [v for k, v in rows if "aa::" not in k]
            if not other:
                return {}, "no calibration dispatch in the %s run" % counter
            scale = (CALIBRATION_BYTES / 1024.0) / max(other)      # counters are in KiB
            pos = 0
            table = {}
            for b in book:
                pos += b["first_call_kernels"]
                n, kps = b["steps"] * b["kernels_per_step"], b["kernels_per_step"]
                seg = lib_rows[pos:pos + n]
                pos += n
                if len(seg) != n:
                    return {}, "dispatch count mismatch in the %s run" % counter
                table[b["workload"]] = [statistics.median(seg[j][1] for j in range(i, n, kps)) * scale * 1024.0
                                        for i in range(kps)]
            per_counter[counter] = (table, scale)
        for w in workloads:
            f, wr = per_counter["FETCH_SIZE"][0].get(w), per_counter["WRITE_SIZE"][0].get(w)
            if f is None or wr is None or len(f) != len(wr):
                continue
            out[w] = [{"hbm_bytes": a + b, "fetch_bytes": a, "write_bytes": b} for a, b in zip(f, wr)]
        note = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in this run; scale factors %.4f / %.4f from a %d MiB copy" % (
            per_counter["FETCH_SIZE"][1], per_counter["WRITE_SIZE"][1], CALIBRATION_BYTES >> 20)
        return out, note
    except (OSError, subprocess.SubprocessError, ValueError, KeyError) as e:
        return {}, "traffic measurement failed: %r" % (e,)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the forward pass of one batch has no cross-GPU part); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.traffic_pass:
        traffic_pass(args)
        return
    names = [args.workload] + ([] if args.no_others else [w for w in ORDER if w != args.workload])
    traffic, traffic_note = ({}, "skipped (--no-traffic)")
    if not args.no_traffic:      # child processes first: this process has not touched the GPU yet
        traffic, traffic_note = measure_traffic(names, args.mode, args.ring_bytes)

    import torch
    from paper_2312_08874_amd import binding, inputs
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    torch.cuda.set_device(0)
    wl = inputs.WORKLOADS[args.workload]
    module = args.mode == "module"

    res, ring = measure(wl, binding, args, args.steps, args.warmup, module, traffic.get(wl.name))
    line = {
        "metric": "agent-attn fwd tokens/s + % of binding roofline (HBM or MFMA), 1 MI355X",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "heads": wl.heads, "N": wl.N, "d": wl.d, "n": wl.n,
                   "mode": args.mode, "cache": "cold (ring of %d input sets)" % res["ring_sets"],
                   "kernels": res["plan"]},
        "tflops": res["tflops"], "path_gbs": res["path_gbs"], "path_roofline_frac": res["path_roofline_frac"],
        "kernels": res["kernels"],
        "roofline": res["roofline"],
        "traffic_source": traffic_note,
    }
    if "path_hbm_bytes_measured" in res:
        line["path_hbm_bytes_measured"] = res["path_hbm_bytes_measured"]
        line["algorithmic_path_bytes"] = res["algorithmic_path_bytes"]
    if args.backward:
        line["backward"] = measure_backward(wl, binding, ring, max(5, args.steps // 15), 3)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, ring)
    del ring
    torch.cuda.empty_cache()
    if not args.no_others:
        # the same workload hot (two input sets, everything stays in the Infinity Cache) and with the other
        # set of module terms (agent bias with 7x7 block components and DWC on / off), cold
        copy_gbs = measured_copy_gbs()
        line["measured_copy_gbs"] = copy_gbs
        k, w = max(30, args.steps // 3), max(5, args.warmup // 3)
        other_mode = "pure" if module else "module"
        line["variants"] = {
            "%s_hot_us" % args.mode: step_time(wl, binding, 1.0, k, w, module) * 1e3,
            "%s_cold_us" % other_mode: step_time(wl, binding, args.ring_bytes, k, w, not module) * 1e3,
            "module_prepared_bias_cold_us": step_time(wl, binding, args.ring_bytes, k, w, True, True) * 1e3,
        }
        line["variants"]["tiny_single_call_latency_us"] = single_call_latency_us(inputs.WORKLOADS["tiny"], binding)
        try:      # two library GEMMs around the operator; not part of the headline figure
            line["variants"]["with_projections_hot_us"] = module_with_projections_us(wl, binding)
        except Exception as e:      # the BLAS library is an optional dependency of that entry point alone
            line["variants"]["with_projections_hot_us"] = None
            line["variants"]["with_projections_note"] = repr(e)[:120]
        others = {}
        for name in names[1:]:
            w2 = inputs.WORKLOADS[name]
            r, rg = measure(w2, binding, args, max(20, args.steps), max(5, args.warmup), module, traffic.get(name))
            r["value"] = r.pop("tokens_per_s")
            r["unit"] = "tokens/s"
            if r["roofline"]["bound"] == "hbm":
                r["roofline"]["frac_of_measured_copy"] = r["roofline"]["achieved"] / copy_gbs
            if not args.no_cpu_baseline:
                r["cpu_baseline"] = cpu_baseline(w2, rg)
            del rg
            torch.cuda.empty_cache()
            others[name] = r
        line["workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
