#!/usr/bin/env python3
"""Benchmark of the agent-attention forward pass on one MI355X.

A step is one pass of the whole hot path (pooling, aggregation + merge, broadcast)
over one batch of seeded synthetic inputs that already sit in HBM.  Steps rotate
over a ring of input/output sets larger than the 256 MB Infinity Cache so that
every step reads its inputs from HBM ("cold").  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload deit_t] [--mode pure|module]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, GB/s
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16 MFMA, TFLOP/s
VALU_F32_PEAK_TFLOPS = 157.3   # fp32 vector arithmetic, published figure, TFLOP/s
ELEM = {"f32": 4, "f16": 2, "bf16": 2}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="deit_t")
    ap.add_argument("--mode", default="pure", choices=["pure", "module"])
    ap.add_argument("--backward", action="store_true",
                    help="also time agent_attn_bwd on the workload and add a \"backward\" object to the line")
    ap.add_argument("--ring-bytes", type=float, default=1.25e9, help="total footprint of the rotating input sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short summary of the other workloads")
    ap.add_argument("--graph", action="store_true",
                    help="replay the steps from a captured HIP graph (one graph = one pass over the ring)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for the HBM byte counters when profiling)")
    return ap.parse_args()


def stage_bytes(wl):
    """Algorithmic HBM bytes per launch of each stage and of the whole path (all units)."""
    s, u = ELEM[wl.dtype], wl.units
    big, small = u * wl.N * wl.d * s, u * wl.n * wl.d
    return {
        "pool": big + small * s,                       # read Q, write A
        "aggregate": 2 * big + small * s + small * 4,  # read K, V, A; write V_A (fp32)
        "broadcast": 2 * big + small * s + small * 4,  # read Q, A, V_A; write O
        "path": 4 * big,                               # read Q, K, V once, write O once
    }


def stage_flops(wl):
    f = 4.0 * wl.N * wl.n * wl.d * wl.units
    return {"pool": 0.0, "aggregate": f, "broadcast": f, "path": 2 * f}


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
        desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, {"f32": 0, "f16": 1, "bf16": 2}[wl.dtype],
                                 wl.grid, wl.agent_grid)
        ws_bytes = binding.workspace_bytes(desc, binding.make_params(self.params))
        per_set = 4 * base["Q"].numel() * base["Q"].element_size() + ws_bytes
        self.R = max(2, min(256, int(ring_bytes // per_set) + 1))
        self.sets = []
        for _ in range(self.R):
            s = {k: v.clone() for k, v in base.items()}
            s["out"] = torch.empty_like(base["Q"])
            s["ws"] = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
            s["A"] = torch.empty((wl.batch, wl.heads, wl.n, wl.d), dtype=base["Q"].dtype, device="cuda")
            s["VA"] = torch.empty((wl.batch, wl.heads, wl.n, wl.d), dtype=torch.float32, device="cuda")
            self.sets.append(s)

        b, p = binding, self.params
        self.fwd = [b.prepare_fwd(s["Q"], s["K"], s["V"], grid=wl.grid, agent_grid=wl.agent_grid, params=p,
                                  out=s["out"], workspace=s["ws"]) for s in self.sets]
        self.stages = {
            "pool": [b.prepare_pool(s["Q"], grid=wl.grid, agent_grid=wl.agent_grid, out=s["A"]) for s in self.sets],
            "aggregate": [b.prepare_aggregate(s["A"], s["K"], s["V"], grid=wl.grid, params=p, out=s["VA"],
                                              workspace=s["ws"]) for s in self.sets],
            "broadcast": [b.prepare_broadcast(s["Q"], s["A"], s["VA"], s["V"], grid=wl.grid, params=p, out=s["out"])
                          for s in self.sets],
        }

    def forward(self, i):
        self.fwd[i % self.R]()

    def stage(self, name, i):
        self.stages[name][i % self.R]()


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


def load_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
        return table[workload][kernel]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def roofline_for(wl, stage_ms, fused_ms=None):
    """Roofline entry of the dominant kernel.

    When the whole step is one kernel (the one-block-per-unit path) that kernel is the entry, with the
    algorithmic bytes of the whole path and the step time as its launch duration.  Otherwise it is the
    stage with the longest average launch (aggregate = split pass + merge, timed together)."""
    if fused_ms is not None:
        name, ms = "path", fused_ms
        label = "small_fused"
    else:
        name = max(stage_ms, key=stage_ms.get)
        ms = stage_ms[name]
        label = name
    traffic = load_traffic(wl.name, label)
    if wl.n >= 1024:
        ach = stage_flops(wl)[name] / (ms * 1e-3) / 1e12
        return {"kernel": label, "bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_PEAK_TFLOPS, "traffic": traffic, "avg_launch_us": ms * 1e3}
    ach = stage_bytes(wl)[name] / (ms * 1e-3) / 1e9
    return {"kernel": label, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": traffic, "avg_launch_us": ms * 1e3}


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


def step_time(wl, binding, ring_bytes, steps, warmup, module, prepared=False):
    """Milliseconds per forward pass alone (no stage timings), for the hot and module-mode variants."""
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
    import statistics
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


def measure(wl, binding, args, steps, warmup, module):
    import torch
    ring = Ring(wl, binding, args.ring_bytes, module)
    ms = timed_graph(ring, steps, warmup) if args.graph else timed(ring.forward, steps, warmup)
    ring.stage("pool", 0)
    ring.stage("aggregate", 0)
    torch.cuda.synchronize()
    stage_ms = {st: timed(lambda i, st=st: ring.stage(st, i), steps, max(3, warmup // 3))
                for st in ("pool", "aggregate", "broadcast")}
    tokens = wl.batch * wl.N
    desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, {"f32": 0, "f16": 1, "bf16": 2}[wl.dtype],
                             wl.grid, wl.agent_grid)
    plan = binding.plan_str(desc)
    res = {
        "ms_per_step": ms,
        "tokens_per_s": tokens / (ms * 1e-3),
        "tflops": stage_flops(wl)["path"] / (ms * 1e-3) / 1e12,
        "path_gbs": stage_bytes(wl)["path"] / (ms * 1e-3) / 1e9,
        "stage_us": {k: v * 1e3 for k, v in stage_ms.items()},
        "roofline": roofline_for(wl, stage_ms, ms if plan == "small_fused" else None),
        "plan": plan,
        "ring_sets": ring.R,
    }
    res["path_roofline_frac"] = (res["tflops"] / MFMA_PEAK_TFLOPS) if wl.n >= 1024 else (res["path_gbs"] / HBM_PEAK_GBS)
    return res, ring


def measure_backward(wl, binding, ring, steps, warmup):
    """agent_attn_bwd on the first input set (same buffers every call: the dense attention matrices in its
    workspace dwarf the inputs, so a cold ring would add nothing).  20*N*n*d FLOPs per unit in ten matrix
    products: on MFMA for fp16 / bf16 (priced against the dense MFMA peak), as fp32 vector FMAs for fp32
    (priced against the fp32 vector peak)."""
    import torch
    s = ring.sets[0]
    dO = torch.randn(s["Q"].shape, device="cuda", dtype=torch.float32).to(s["Q"].dtype)
    desc = binding.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, {"f32": 0, "f16": 1, "bf16": 2}[wl.dtype],
                             wl.grid, wl.agent_grid)
    import ctypes
    need = int(binding.lib().agent_attn_bwd_workspace_bytes(ctypes.byref(desc), binding._pp(binding.make_params(ring.params))))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def call(i):
        binding.agent_attn_bwd(s["Q"], s["K"], s["V"], dO, grid=wl.grid, agent_grid=wl.agent_grid, params=ring.params,
                               workspace=ws)
    ms = timed(call, steps, warmup)
    flops = 20.0 * wl.N * wl.n * wl.d * wl.units
    tf = flops / (ms * 1e-3) / 1e12
    peak = VALU_F32_PEAK_TFLOPS if wl.dtype == "f32" else MFMA_PEAK_TFLOPS
    return {"ms_per_step": ms, "tokens_per_s": wl.batch * wl.N / (ms * 1e-3), "tflops": tf,
            "workspace_bytes": need, "cache": "hot (one input set)",
            "kernels": "reference-quality: 10 batched matrix products + row softmax / gradient kernels, attention "
                       "matrices materialised in the workspace",
            "roofline": {"kernel": "matmul_kernel" if wl.dtype == "f32" else "mfma_matmul_kernel",
                         "bound": "alu" if wl.dtype == "f32" else "mfma", "achieved": tf, "peak": peak,
                         "unit": "TFLOP/s", "frac": tf / peak, "traffic": None}}


def cpu_baseline(wl, ring):
    """The fp64 oracle, as it stands, on the host cores: a bounded sample of the same workload."""
    from oracle import agent_attn_oracle as oracle
    from paper_2312_08874_amd import inputs
    from tests import util
    flops_unit = 8.0 * wl.N * wl.n * wl.d
    units = int(max(1, min(wl.units, 1.2e10 // flops_unit)))
    t = {k: v[:units] for k, v in ring.host.items()}
    q, k, v = (inputs.to_float64(t[x], wl.dtype) for x in ("Q", "K", "V"))
    kw = {}
    if ring.host_params:
        B1, B2 = util.dense_biases(oracle, ring.host_params, wl.heads, wl.n, wl.grid)
        kw = dict(B1=B1, B2=B2, dwc_w=ring.host_params["dwc_w"], dwc_b=ring.host_params["dwc_b"])
    heads = wl.heads if units % wl.heads == 0 else 1
    if heads == 1 and kw:
        kw = {kk: vv[:1] for kk, vv in kw.items()}
    oracle.agent_attn_fwd(q[:1], k[:1], v[:1], heads=1, grid=wl.grid, agent_grid=wl.agent_grid,
                          **({kk: vv[:1] for kk, vv in kw.items()}))      # warm the library
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < 1.5 and reps < 200:          # about 1.5 s of wall time on all host cores
        oracle.agent_attn_fwd(q, k, v, heads=heads, grid=wl.grid, agent_grid=wl.agent_grid, **kw)
        reps += 1
        dt = time.perf_counter() - t0
    tokens = reps * units * wl.N / wl.heads
    return {"value": tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d (batch*head) units of workload %s, fp64, %d repetition(s), %.2f s wall"
                      % (units, wl.units, wl.name, reps, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the forward pass of one batch has no cross-GPU part); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2312_08874_amd import binding, inputs
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    torch.cuda.set_device(0)
    wl = inputs.WORKLOADS[args.workload]
    module = args.mode == "module"

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    torch.cuda.synchronize()
    res, ring = measure(wl, binding, args, args.steps, args.warmup, module)
    line = {
        "metric": "agent-attn fwd tokens/s + % of binding roofline (HBM or MFMA), 1 MI355X",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "heads": wl.heads, "N": wl.N, "d": wl.d, "n": wl.n,
                   "mode": args.mode, "cache": "cold (ring of %d input sets)" % res["ring_sets"],
                   "kernels": res["plan"]},
        "tflops": res["tflops"], "path_gbs": res["path_gbs"], "path_roofline_frac": res["path_roofline_frac"],
        "stage_us": res["stage_us"],
        "roofline": res["roofline"],
    }
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
        if line["roofline"]["bound"] == "hbm":
            line["roofline"]["frac_of_measured_copy"] = line["roofline"]["achieved"] / copy_gbs
        k, w = max(50, args.steps // 3), max(5, args.warmup // 3)
        other_mode = "pure" if module else "module"
        line["variants"] = {
            "%s_hot_us" % args.mode: step_time(wl, binding, 1.0, k, w, module) * 1e3,
            "%s_cold_us" % other_mode: step_time(wl, binding, args.ring_bytes, k, w, not module) * 1e3,
            "%s_hot_us" % other_mode: step_time(wl, binding, 1.0, k, w, not module) * 1e3,
            "module_prepared_bias_cold_us": step_time(wl, binding, args.ring_bytes, k, w, True, True) * 1e3,
        }
        line["variants"]["tiny_single_call_latency_us"] = single_call_latency_us(inputs.WORKLOADS["tiny"], binding)
        others = {}
        for name, w in inputs.WORKLOADS.items():
            if name == wl.name:
                continue
            r, rg = measure(w, binding, args, max(20, args.steps // 3), max(5, args.warmup // 3), module)
            del rg
            torch.cuda.empty_cache()
            others[name] = {"tokens_per_s": r["tokens_per_s"], "ms_per_step": r["ms_per_step"], "tflops": r["tflops"],
                            "path_gbs": r["path_gbs"], "path_roofline_frac": r["path_roofline_frac"],
                            "stage_us": r["stage_us"], "kernels": r["plan"], "dominant": r["roofline"]["kernel"],
                            "dominant_frac": r["roofline"]["frac"]}
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
