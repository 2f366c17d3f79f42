#!/usr/bin/env python3
"""Benchmark of the operator-split linear layer (libosdp) on one MI355X.

Default workload: the wide feed-forward pair of the benchmark's configs[3] (h = 8192, 4096 tokens), the one
whose slice granularity the metric sweeps ("vs k; peak staging MB").

A step is one pass of the whole hot path over one batch of synthetic input:
for every operator of the workload, the split forward (gather slice j, slice
GEMM) and then, in reverse operator order, the split backward (gather again,
dW slice GEMM, dX accumulate GEMM).  Inputs are resident in HBM before the
timed region starts.

Prints one JSON line: whole-job TFLOP/s (6*T*I*O flops per operator), the
roofline of the dominant kernel measured with HIP events inside this run, and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (vendor figure: 256 CUs x 2.4 GHz x 4096 flop/clk/CU)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak

# HBM-side traffic per launch of each GEMM kind, from the rocprofv3 --pmc summaries under profiles/ (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for plain copies of known size): lines of the form
# "traffic_bytes_per_launch <kernel kind> <bytes>" in profiles/hbm_traffic_config<N>.md.  None where no summary exists.
def measured_traffic(config, kind):
    import re
    from pathlib import Path
    f = Path(__file__).resolve().parent / "profiles" / f"hbm_traffic_config{config}.md"
    if not f.exists():
        return None
    m = re.search(rf"^traffic_bytes_per_launch\s+{kind}\s+(\d+)", f.read_text(), re.M)
    return int(m.group(1)) if m else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="workload: index into BASELINE.json configs (1-based)")
    ap.add_argument("--k", type=int, default=None, help="slice granularity (default: the workload's own)")
    ap.add_argument("--staging", choices=["auto", "single", "double", "half"], default="auto")
    ap.add_argument("--split-dim", choices=["out", "in", "longer", "perpass"], default="out",
                    help="cut W along its output features (columns), its input features (rows, the reduction "
                         "dimension), per operator along the longer of the two, or along the columns in the forward pass and "
                         "the rows in the backward pass (no fp32 partial sum in either)")
    ap.add_argument("--zdp-slices", type=int, default=None,
                    help="keep only the first Z slices of every operator sharded (ZDP); the others are DP slices "
                         "read from a resident replica (default: every slice ZDP)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the k x staging sweep and the other workloads")
    ap.add_argument("--gathers", choices=["carried", "launched"], default="carried",
                    help="carried: a GEMM launch takes the next slice's gather along (the library's default); launched: "
                         "every gather is a kernel launch of its own, on the copy stream where the pipeline overlaps")
    ap.add_argument("--no-auto", action="store_true", help="skip the automatic slice-granularity table")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="first run three plain copies of 1 GiB through the gather kernel (one shard, one slice, source "
                         "far larger than every cache): the known traffic that HBM counters of a profiled run are scaled by")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--serial", action="store_true", help="one stream: no gather/GEMM overlap")
    return ap.parse_args()


class Stack:
    """All operators of a workload resident on the GPU, with one shared workspace."""

    def __init__(self, w, staging, torch, osdp, seed=0, rows=False, plan=None, zdp_slices=None, zdp_masks=None,
                 longer=False, per_pass=False):
        self.w, self.torch, self.osdp = w, torch, osdp
        g = torch.Generator(device="cuda")
        g.manual_seed(220913258 + seed)
        bf = torch.bfloat16
        self.ops = []
        for layer in range(w.layers):
            for n, op in enumerate(w.ops):
                L = -(-(op.I * op.O) // w.N)
                d = dict(
                    n=n, op=op,
                    X=torch.randn((w.T, op.I), generator=g, device="cuda", dtype=torch.float32).to(bf),
                    dY=torch.randn((w.T, op.O), generator=g, device="cuda", dtype=torch.float32).to(bf),
                    W=[(torch.randn((L,), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(bf) for _ in range(w.N)],
                    Y=torch.empty((w.T, op.O), device="cuda", dtype=bf),
                    dX=torch.empty((w.T, op.I), device="cuda", dtype=bf),
                    dW=[torch.empty((L,), device="cuda", dtype=bf) for _ in range(w.N)],
                )
                self.ops.append(d)
        dims = [osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES] * len(w.ops)
        if longer:
            dims = [osdp.OSDP_SPLIT_LONGER] * len(w.ops)
        if per_pass:
            dims = [osdp.OSDP_SPLIT_PER_PASS] * len(w.ops)
        self.plan = plan or osdp.Plan([op.k for op in w.ops], staging=staging, split_dim_per_op=dims)
        # zdp_slices = z: the first z slices of every operator stay sharded (ZDP), the others are DP slices read from
        # a resident full-layout replica, their gradients written to a full-layout array
        self.mixed = zdp_slices is not None or zdp_masks is not None
        if self.mixed:
            self.plan.zdp_mask = list(zdp_masks) if zdp_masks is not None else \
                [(1 << min(zdp_slices, max(op.k, 1))) - 1 for op in w.ops]
            for d in self.ops:
                op, k = d["op"], max(d["op"].k, 1)
                d["Wfull"] = (torch.randn((op.I * op.O,), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(bf)
                d["dWfull"] = torch.empty((op.I * op.O,), device="cuda", dtype=bf)
                starts = [(j * op.I // k) * op.O if rows else j * op.O // k for j in range(k)]
                mask = self.plan.zdp_mask[d["n"]]
                d["w_dp"] = [None if (mask >> j) & 1 else d["Wfull"][s:] for j, s in enumerate(starts)]
                d["dw_dp"] = [None if (mask >> j) & 1 else d["dWfull"][s:] for j, s in enumerate(starts)]
        need, self.peak_staging = 0, 0
        for n, op in enumerate(w.ops):
            for is_bwd in (False, True):
                tot, peak = osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, 0, is_bwd, self.plan, n)
                need, self.peak_staging = max(need, tot), max(self.peak_staging, peak)
        self.workspace_bytes = need
        self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        self.sc, self.sp = torch.cuda.Stream(), torch.cuda.Stream()

    def step(self, serial=False):
        osdp, sp = self.osdp, (None if serial else self.sp)
        if self.mixed:
            for d in self.ops:
                osdp.osdp_split_linear_fwd_mixed(d["X"], d["W"], d["w_dp"], d["op"].O, d["Y"], 0, self.ws, plan=self.plan,
                                                 op_index=d["n"], stream_compute=self.sc, stream_copy=sp)
            for d in reversed(self.ops):
                osdp.osdp_split_linear_bwd_mixed(d["X"], d["dY"], d["W"], d["w_dp"], d["op"].O, d["dX"], d["dW"],
                                                 d["dw_dp"], 0, self.ws, plan=self.plan, op_index=d["n"],
                                                 stream_compute=self.sc, stream_copy=sp)
            return
        for d in self.ops:
            osdp.osdp_split_linear_fwd(d["X"], d["W"], d["Y"], 0, self.ws, plan=self.plan, op_index=d["n"],
                                       stream_compute=self.sc, stream_copy=sp)
        for d in reversed(self.ops):
            osdp.osdp_split_linear_bwd(d["X"], d["dY"], d["W"], d["dX"], d["dW"], 0, self.ws, plan=self.plan,
                                       op_index=d["n"], stream_compute=self.sc, stream_copy=sp)

    def run(self, steps, warmup, serial=False, profile=False):
        """Returns (ms per step, per-kernel stats or None)."""
        torch, osdp = self.torch, self.osdp
        with torch.cuda.stream(self.sc):
            for _ in range(warmup):
                self.step(serial)
            torch.cuda.synchronize()
            if profile:
                osdp.osdp_profile_begin(1 << 20)
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step(serial)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            stats = osdp.osdp_profile_end() if profile else None
            if profile:
                stats["_overlap"] = osdp.osdp_profile_overlap()
        return (t1 - t0) * 1e3 / steps, stats


def per_step_times(st, iters, warmup, serial):
    """Each step timed on its own by a pair of HIP events on the compute stream: (median ms, mean ms)."""
    torch = st.torch
    with torch.cuda.stream(st.sc):
        for _ in range(warmup):
            st.step(serial)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for e0, e1 in ev:
            e0.record(st.sc)
            st.step(serial)
            e1.record(st.sc)
        torch.cuda.synchronize()
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    return ms[len(ms) // 2], sum(ms) / len(ms)


def graph_replay_ms(st, iters, warmup):
    """One step captured into a HIP graph on the compute stream (the cross-stream edges of the two-stream pipeline
    inside the capture), then replayed: median ms per replay.  What the launch gaps of the eager step cost."""
    torch = st.torch
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st.sc):
        st.step(False)
    with torch.cuda.stream(st.sc):
        for _ in range(warmup):
            graph.replay()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for e0, e1 in ev:
            e0.record(st.sc)
            graph.replay()
            e1.record(st.sc)
        torch.cuda.synchronize()
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    del graph
    return ms[len(ms) // 2]


def library_vs_vendor_gemm(torch, osdp, size=8192, reps=10):
    """The three GEMM layouts of the path on one cube, library launches (k = 1, timed by the library's own events)
    beside torch.matmul (the vendor GEMM library) on the same box in the same process: context for the roofline
    fractions, since boxes and their power limits differ."""
    T = I = O = size
    N = 8
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    X = torch.randn(T, I, generator=g, device="cuda").to(torch.bfloat16)
    dY = torch.randn(T, O, generator=g, device="cuda").to(torch.bfloat16)
    Wd = (torch.randn(I, O, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    L = I * O // N
    W = [Wd.reshape(-1)[s * L:(s + 1) * L].clone() for s in range(N)]
    dW = [torch.empty(L, dtype=torch.bfloat16, device="cuda") for _ in range(N)]
    Y = torch.empty(T, O, dtype=torch.bfloat16, device="cuda")
    dX = torch.empty(T, I, dtype=torch.bfloat16, device="cuda")
    plan = osdp.Plan([1])
    need = max(osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, b, plan, 0)[0] for b in (False, True))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    sc = torch.cuda.Stream()
    with torch.cuda.stream(sc):
        for rep in range(2):
            if rep == 1:
                osdp.osdp_profile_begin()
            for _ in range(reps if rep else 3):
                osdp.osdp_split_linear_fwd(X, W, Y, 1, ws, plan=plan, stream_compute=sc)
                osdp.osdp_split_linear_bwd(X, dY, W, dX, dW, 1, ws, plan=plan, stream_compute=sc)
            sc.synchronize()
        st = osdp.osdp_profile_end()
    flops = 2.0 * size ** 3
    lib = {kind: round(flops / (st[name]["ms"] / st[name]["launches"] * 1e-3) / 1e12, 1)
           for kind, name in (("fwd_nn", "gemm_fwd"), ("dx_nt", "gemm_dx"), ("dw_tn", "gemm_dw"))}

    def vendor(fn):
        for _ in range(3):
            fn()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in ev:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)[reps // 2]
        return round(flops / (ms * 1e-3) / 1e12, 1)
    ven = {"fwd_nn": vendor(lambda: torch.matmul(X, Wd)), "dx_nt": vendor(lambda: torch.matmul(dY, Wd.t())),
           "dw_tn": vendor(lambda: torch.matmul(X.t(), dY))}
    return {"shape": [size, size, size], "library_tflops": lib, "torch_matmul_tflops": ven,
            "note": "library: per-launch HIP events around each kernel; torch.matmul: events around each call, median"}


def kernel_table(stats):
    out = {}
    for name, s in stats.items():
        if name.startswith("_") or not s["launches"]:
            continue
        if name == "gather_carried":   # gathers that ran inside GEMM launches: no time of their own
            out[name] = dict(launches=s["launches"], mb=round(s["bytes"] / 2 / 2 ** 20, 2))
            continue
        if name == "gemm_persistent":  # GEMM launches (counted under their kinds) that ran as the persistent kernel
            out[name] = dict(launches=s["launches"])
            continue
        avg_ms = s["ms"] / s["launches"]
        e = dict(launches=s["launches"], avg_us=round(avg_ms * 1e3, 2), total_ms=round(s["ms"], 3))
        if s["flops"]:
            e["tflops"] = round(s["flops"] / (s["ms"] * 1e-3) / 1e12, 2)
            e["frac_mfma_peak"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
        e["gbs_algorithmic"] = round(s["bytes"] / (s["ms"] * 1e-3) / 1e9, 1)
        out[name] = e
    return out


def measure(st, flops, steps, warmup, serial, config=None):
    """The figures of one resident stack: median and mean of `steps` individually timed steps, the per-kernel table of a
    second, instrumented pass of the same steps (every launch bracketed by HIP events on its own stream), the roofline
    of the GEMM kind with the largest summed time, and where the gathers went."""
    median_ms, mean_ms = per_step_times(st, steps, warmup, serial)
    n_prof = max(10, steps // 2)
    ms_prof, stats = st.run(n_prof, 2, serial=serial, profile=True)
    ov = stats["_overlap"]
    kernels = kernel_table(stats)
    gemms = {k: v for k, v in kernels.items() if k.startswith("gemm") and "total_ms" in v}
    dom = max(gemms, key=lambda k: gemms[k]["total_ms"])
    roofline = {"bound": "mfma", "kernel": dom, "achieved": gemms[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(gemms[dom]["tflops"] / PEAK_BF16_TFLOPS, 4),
                "traffic": measured_traffic(config, dom) if config else None,
                "algorithmic_bytes": round(stats[dom]["bytes"] / stats[dom]["launches"]),
                "avg_launch_us": gemms[dom]["avg_us"], "launches_per_step": gemms[dom]["launches"] // n_prof}
    g, c = kernels.get("gather"), kernels.get("gather_carried")
    gathers = {"launched_per_step": (g["launches"] // n_prof) if g else 0,
               "launched_us_per_step": round(g["total_ms"] * 1e3 / n_prof, 1) if g else 0.0,
               "launched_gbs": g["gbs_algorithmic"] if g else None,
               "launched_frac_hbm_peak": round(g["gbs_algorithmic"] / PEAK_HBM_GBS, 4) if g else None,
               "carried_by_gemm_launches_per_step": (c["launches"] // n_prof) if c else 0,
               "carried_mb_per_step": round(c["mb"] / n_prof, 2) if c else 0.0,
               # time in which a gather kernel ran and no GEMM did (instrumented pass, all streams on one clock)
               "exposed_us_per_step": round(ov["gather_exposed_ms"] * 1e3 / n_prof, 1)}
    tf = flops / (median_ms * 1e-3) / 1e12
    return {"tflops": round(tf, 2), "frac_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4),
            "median_ms_per_step": round(median_ms, 4), "mean_ms_per_step": round(mean_ms, 4), "timed_steps": steps,
            "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3), "workspace_mb": round(st.workspace_bytes / 2 ** 20, 3),
            "roofline": roofline, "gathers": gathers,
            # instrumented pass: the part of a step in which no kernel of the library ran (launch gaps, event handling)
            "idle_us_per_step": round(ov["idle_ms"] * 1e3 / n_prof, 1),
            "kernels": kernels}


def auto_granularity(st, osdp, torch, steps, warmup):
    """Every (k, split dimension, staging) candidate of each operator timed by the library on the stack's own
    buffers, and what the selection rule picks: fastest overall, least gathered weight within 10 % of it, and the
    fastest within the peak staging of the stack's own plan; the step is then timed under that last choice."""
    names = {osdp.OSDP_STAGING_SINGLE: "single", osdp.OSDP_STAGING_DOUBLE: "double", osdp.OSDP_STAGING_HALF: "half"}
    out, picked = {}, []
    for d in st.ops[:len(st.w.ops)]:
        op = d["op"]
        cands = osdp.osdp_granularity_candidates(st.w.T, op.I, op.O, st.w.N, [1, 2, 4, 8, 16])
        ws = torch.empty(max(c.workspace for c in cands), dtype=torch.uint8, device="cuda")
        with torch.cuda.stream(st.sc):
            osdp.osdp_granularity_measure(d["X"], d["dY"], d["W"], d["Y"], d["dX"], d["dW"], ws, cands, warmup=2, reps=5,
                                          stream_compute=st.sc, stream_copy=st.sp)
        torch.cuda.synchronize()

        def show(i):
            c = cands[i]
            return {"k": c.k, "split_dim": {0: "out", 1: "in", 3: "per_pass"}[c.split_dim], "staging": names[c.staging],
                    "peak_staging_mb": round(c.peak_weight_staging / 2 ** 20, 3), "workspace_mb": round(c.workspace / 2 ** 20, 3),
                    "ms": round(c.ms, 4), "tflops": round(6 * st.w.T * op.I * op.O / (c.ms * 1e-3) / 1e12, 1)}
        same_budget = osdp.osdp_granularity_select(cands, st.peak_staging, 0, 0.0)
        picked.append(cands[same_budget])
        out[op.name] = {"candidates": len(cands),
                        "fastest": show(osdp.osdp_granularity_select(cands, 0, 0, 0.0)),
                        "fastest_within_default_peak_staging": show(same_budget),
                        "least_staging_within_10pct": show(osdp.osdp_granularity_select(cands, 0, 0, 0.10)),
                        "table": [show(i) for i in range(len(cands))]}
    # the whole step under the per-operator choices
    plan = osdp.Plan([c.k for c in picked], split_dim_per_op=[c.split_dim for c in picked],
                     staging_per_op=[c.staging for c in picked])
    tuned = Stack(st.w, 0, torch, osdp, plan=plan)
    ms = per_step_times(tuned, steps, warmup, False)[0]   # median of individually timed steps
    import workloads as wl
    out["step_under_chosen_plan"] = {"k_per_op": list(plan.k_per_op), "split_dim_per_op": list(plan.split_dim_per_op),
                                     "staging_per_op": [names[m] for m in plan.staging_per_op], "ms_per_step": round(ms, 4),
                                     "tflops": round(wl.flops(st.w) / (ms * 1e-3) / 1e12, 2),
                                     "peak_staging_mb": round(tuned.peak_staging / 2 ** 20, 3),
                                     "workspace_mb": round(tuned.workspace_bytes / 2 ** 20, 3)}
    return out


def measure_alpha(torch, osdp, reps=200):
    """Fixed cost of one gather, in seconds: the smallest legal slice (8 x 8 elements from one shard) copied `reps`
    times back to back on one stream, timed by a pair of events."""
    shard = [torch.zeros(64, dtype=torch.bfloat16, device="cuda")]
    stg = torch.empty(64, dtype=torch.bfloat16, device="cuda")
    cur = torch.cuda.current_stream()
    for _ in range(10):
        osdp.osdp_split_linear_gather_slice(8, 8, 1, 0, shard, stg, stream=cur)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(cur)
    for _ in range(reps):
        osdp.osdp_split_linear_gather_slice(8, 8, 1, 0, shard, stg, stream=cur)
    e1.record(cur)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def plan_search(w, kernels, staging, rows, torch, osdp, steps, warmup):
    """Algorithm 1 on this workload with device information taken from this run: every slice of every operator is
    an item (Section 3.3), gamma from the measured GEMM throughput, beta from the measured gather bandwidth, alpha
    from the measured fixed cost of the smallest gather; the memory limit leaves room for half of the weights to be replicated.
    The chosen per-slice modes are then run through the mixed entry points and timed."""
    import workloads as wl
    gemm_ms = sum(v["total_ms"] for k, v in kernels.items() if k.startswith("gemm") and "total_ms" in v)
    gemm_flops = sum(v["tflops"] * v["total_ms"] for k, v in kernels.items() if k.startswith("gemm") and "total_ms" in v) * 1e9
    flops_per_s = gemm_flops / (gemm_ms * 1e-3)
    gather = kernels.get("gather")
    beta = 1.0 / (gather["gbs_algorithmic"] * 1e9 / 2) if gather else 1.0 / 2e12   # seconds per byte gathered
    alpha = measure_alpha(torch, osdp)
    items, owner = [], []
    for layer in range(w.layers):
        for n, op in enumerate(w.ops):
            k = max(op.k, 1)
            for j in range(k):
                size = op.I * op.O * 2 / k
                # model states = the bf16 weights and their gradient; no activations are kept by this path
                items.append((2 * size, 0.0, 0.0, size, 6.0 * op.I * op.O / k / flops_per_s))
                owner.append((layer, n, j))
    limit = 0.5 * sum(i[0] for i in items) * (1 + 1 / w.N)
    t0 = time.perf_counter()
    r = osdp.osdp_plan_search(items, w.N, alpha, beta, limit, b_max=w.T)
    search_ms = (time.perf_counter() - t0) * 1e3
    if r is None:
        return {"found": False, "search_ms": round(search_ms, 3)}
    masks = [0] * len(w.ops)   # the stack shares one plan over its layers: take the first layer's modes
    for (layer, n, j), m in zip(owner, r["modes"]):
        if layer == 0 and m:
            masks[n] |= 1 << j
    st = Stack(w, staging, torch, osdp, rows=rows, zdp_masks=masks)
    ms = per_step_times(st, steps, warmup, False)[0]   # median of individually timed steps
    return {"found": True, "items": len(items), "memory_limit_mb": round(limit / 2 ** 20, 3),
            "device_info": {"alpha_s": alpha, "beta_s_per_byte": beta, "gemm_flops_per_s": flops_per_s},
            "zdp_mask_per_op": {op.name: bin(m) for op, m in zip(w.ops, masks)}, "zdp_items": int(sum(r["modes"])),
            "model_memory_mb": round(r["memory"] / 2 ** 20, 3), "search_ms": round(search_ms, 3),
            "plans_visited": r["plans_visited"], "exact": r["exact"], "batch_sizes_tried": r["batch_sizes_tried"],
            "measured_ms_per_step": round(ms, 4), "measured_tflops": round(wl.flops(w) / (ms * 1e-3) / 1e12, 2),
            "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3)}


def cpu_baseline(w, target_s=15.0, rows=False):
    """The oracle's split route on a token sub-sample of the same workload, all host threads."""
    import numpy as np
    import oracle
    import workloads as wl

    def one_pass(Ts):
        fl, t = 0, 0.0
        for n, op in enumerate(w.ops):
            d = wl.operator_inputs(w.cfg, 0, n, Ts, op.I, op.O, w.N)
            t0 = time.perf_counter()
            if rows:
                oracle.split_fwd_rows(d["X"], d["W_shards"], op.O, op.k)
                oracle.split_bwd_rows(d["X"], d["dY"], d["W_shards"], op.O, op.k)
            else:
                oracle.split_fwd(d["X"], d["W_shards"], op.O, op.k)
                oracle.split_bwd(d["X"], d["dY"], d["W_shards"], op.O, op.k)
            t += time.perf_counter() - t0
            fl += 6 * Ts * op.I * op.O
        return fl, t

    oracle.build()
    per_token = sum(6 * op.I * op.O for op in w.ops)
    Ts, fl, t = 16, 0, 0.0
    for _ in range(3):                        # grow the sample until one pass takes about target_s
        fl, t = one_pass(Ts)
        if t >= 0.5 * target_s or Ts >= w.T:
            break
        rate = fl / max(t, 1e-9)
        Ts = int(min(w.T, max(2 * Ts, target_s * rate / per_token))) // 16 * 16
    return {"value": round(fl / t / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first layer of the workload with T'={Ts} of {w.T} tokens (flops are linear in T), "
                      f"split route fwd+bwd, {t:.1f} s of CPU work"}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build covers one GPU's share of the step; --gpus must be 1 "
              "(no collectives or cross-GPU sharding are part of it)", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    import __graft_entry__
    __graft_entry__.ensure_built()   # loads the library the tree holds; builds one only when there is none
    import paper_2209_13258_amd as osdp
    import workloads as wl

    modes = {"auto": osdp.OSDP_STAGING_AUTO, "single": osdp.OSDP_STAGING_SINGLE,
             "double": osdp.OSDP_STAGING_DOUBLE, "half": osdp.OSDP_STAGING_HALF}
    staging = modes[a.staging]
    osdp.osdp_debug_option("fused_gather", -1 if a.gathers == "carried" else 0)
    if a.traffic_calibration:
        I, O = 16384, 32768   # 1 GiB of bf16
        src = torch.zeros(I * O, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty(I * O, dtype=torch.bfloat16, device="cuda")
        for _ in range(3):
            osdp.osdp_split_linear_gather_slice(I, O, 1, 0, [src], dst)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    w = wl.workload(a.config, a.k)
    rows = a.split_dim == "in"
    longer = a.split_dim == "longer"
    per_pass = a.split_dim == "perpass"
    st = Stack(w, staging, torch, osdp, rows=rows, zdp_slices=a.zdp_slices, longer=longer, per_pass=per_pass)
    flops = wl.flops(w)
    default_plan = a.k is None and a.staging == "auto" and not a.serial and not rows and not longer and not per_pass and \
        a.zdp_slices is None and a.gathers == "carried"

    # ---- the headline: exactly --steps steps after --warmup, one timed region, inputs resident ------------
    torch.cuda.synchronize()
    alloc_before = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    ms, _ = st.run(a.steps, a.warmup, serial=a.serial)
    alloc_delta = torch.cuda.max_memory_allocated() - alloc_before   # the library allocates nothing: the workspace is all
    # individually timed steps: 100 after the warm-up, the paper's protocol (Section 4.1), unless fewer steps were asked for
    n_timed = 100 if a.steps >= 40 else max(a.steps, 20)
    m = measure(st, flops, n_timed, a.warmup, a.serial, config=a.config if default_plan else None)

    out = {
        "metric": "split-linear fwd+bwd TFLOP/s & % bf16 MFMA peak vs k; peak staging MB",
        "value": round(flops / (ms * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "baseline_config": a.config, "T": w.T, "N_shards": w.N, "layers": w.layers,
                   "ops": {op.name: {"I": op.I, "O": op.O, "k": op.k} for op in w.ops},
                   "staging": a.staging, "streams": 1 if a.serial else 2, "gathers": a.gathers,
                   "split_dim": "longer" if longer else "per_pass" if per_pass else "in_features" if rows else "out_features",
                   "zdp_slices": "all" if a.zdp_slices is None else a.zdp_slices},
        "frac_bf16_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "peak_staging_mb": m["peak_staging_mb"], "workspace_mb": m["workspace_mb"],
        "per_step_events": {"iters": m["timed_steps"], "warmup": a.warmup, "median_ms": m["median_ms_per_step"],
                            "mean_ms": m["mean_ms_per_step"]},
        "device_memory_allocated_during_steps_bytes": int(alloc_delta),
        "roofline": m["roofline"], "gathers": m["gathers"], "idle_us_per_step": m["idle_us_per_step"],
        "kernels": m["kernels"],
        # steps of the headline workload run so far (warm-up, timed region, individually timed steps, instrumented
        # pass): what a kernel trace of `--no-sweep --no-auto` divides by
        "headline_steps_executed": a.warmup + a.steps + a.warmup + n_timed + 2 + max(10, n_timed // 2),
    }
    sub_steps, sub_warm = max(20, a.steps // 2), max(3, a.warmup // 2)
    if not a.serial and a.zdp_slices is None:
        # the same step captured into a HIP graph and replayed: what the eager step's launch gaps cost
        mg = graph_replay_ms(st, max(a.steps, 20), a.warmup)
        out["graph_replay"] = {"tflops": round(flops / (mg * 1e-3) / 1e12, 2), "median_ms_per_step": round(mg, 4)}
        out["headline_steps_executed"] += a.warmup + max(a.steps, 20)   # the replays run the step's kernels too

    if not a.no_sweep and a.zdp_slices is None:
        # the gather kernel on its own: one slice of the first operator, back to back (achieved HBM rate of the copy)
        op0 = w.ops[0]
        k0 = max(op0.k, 1)
        stg = torch.empty(op0.I * (op0.O // k0), dtype=torch.bfloat16, device="cuda")
        cur = torch.cuda.current_stream()
        for _ in range(3):
            osdp.osdp_split_linear_gather_slice(op0.I, op0.O, k0, 0, st.ops[0]["W"], stg, stream=cur)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for e0, e1 in ev:
            e0.record(cur)
            osdp.osdp_split_linear_gather_slice(op0.I, op0.O, k0, 0, st.ops[0]["W"], stg, stream=cur)
            e1.record(cur)
        torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) for e0, e1 in ev)[len(ev) // 2]
        gbs = 2 * stg.numel() * 2 / (t * 1e-3) / 1e9
        out["gather_kernel_alone"] = {"slice_mb": round(stg.numel() * 2 / 2 ** 20, 2), "median_us": round(t * 1e3, 2),
                                      "gbs_read_plus_write": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}
        del stg

    if not a.no_sweep and a.zdp_slices is None:
        # Section 4.3, slice granularity: every k of the workload's sweep under every staging mode (column slices, gathers
        # carried by the GEMM launches), then the same k with every operator cut along its longer dimension, with the
        # columns cut in the forward pass and the rows in the backward pass, and with every gather a launch of its own
        # on the copy stream (the two-stream pipeline)
        sweep = {}
        ks = tuple(w.k_sweep or ())
        if ks and 1 not in ks:
            ks = (1,) + ks   # the unsplit operator (the whole weight staged): what every k is set against
        for k in ks:
            wk = wl.workload(a.config, k)
            fk = wl.flops(wk)
            row = {}
            for mname in ("single", "double", "half"):
                if k == 1 and mname != "single":
                    continue
                del st
                torch.cuda.empty_cache()
                st = Stack(wk, modes[mname], torch, osdp, rows=rows)
                mk = measure(st, fk, sub_steps, sub_warm, a.serial)
                row[mname] = {key: mk[key] for key in ("tflops", "frac_bf16_mfma_peak", "median_ms_per_step", "peak_staging_mb",
                                                       "workspace_mb", "gathers", "idle_us_per_step")}
                row[mname]["roofline_frac"] = {kk: vv.get("frac_mfma_peak") for kk, vv in mk["kernels"].items() if kk.startswith("gemm") and "frac_mfma_peak" in vv}
            if k > 1:
                del st
                torch.cuda.empty_cache()
                st = Stack(wk, modes["double"], torch, osdp, longer=True)
                ml = per_step_times(st, sub_steps, sub_warm, a.serial)[0]
                row["double_longer_split_dim"] = {"tflops": round(fk / (ml * 1e-3) / 1e12, 2), "median_ms_per_step": round(ml, 4),
                                                  "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3),
                                                  "workspace_mb": round(st.workspace_bytes / 2 ** 20, 3)}
                del st
                torch.cuda.empty_cache()
                st = Stack(wk, modes["double"], torch, osdp, per_pass=True)
                mp = per_step_times(st, sub_steps, sub_warm, a.serial)[0]
                row["double_per_pass_split_dim"] = {"tflops": round(fk / (mp * 1e-3) / 1e12, 2), "median_ms_per_step": round(mp, 4),
                                                    "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3),
                                                    "workspace_mb": round(st.workspace_bytes / 2 ** 20, 3)}
                del st
                torch.cuda.empty_cache()
                osdp.osdp_debug_option("fused_gather", 0)
                st = Stack(wk, modes["double"], torch, osdp, rows=rows)
                m2 = measure(st, fk, sub_steps, sub_warm, False)
                osdp.osdp_debug_option("fused_gather", -1 if a.gathers == "carried" else 0)
                row["double_gathers_launched_two_streams"] = {key: m2[key] for key in ("tflops", "median_ms_per_step", "gathers", "idle_us_per_step")}
                # the same stack with the persistent form of the four-wave kernel switched off (one tile per workgroup)
                osdp.osdp_debug_option("persistent", 0)
                m3 = per_step_times(st, sub_steps, sub_warm, a.serial)[0]
                osdp.osdp_debug_option("persistent", -1)
                m4 = per_step_times(st, sub_steps, sub_warm, a.serial)[0]
                row["double_one_tile_per_workgroup"] = {"tflops": round(fk / (m3 * 1e-3) / 1e12, 2), "median_ms_per_step": round(m3, 4),
                                                        "persistent_again_tflops": round(fk / (m4 * 1e-3) / 1e12, 2)}
            sweep[str(k)] = row
        if "1" in sweep:   # time(k) / time(unsplit): what splitting costs, overlap and all
            t1 = sweep["1"]["single"]["median_ms_per_step"]
            for row in sweep.values():
                for entry in row.values():
                    entry["time_vs_unsplit"] = round(entry["median_ms_per_step"] / t1, 4)
        out["k_sweep"] = sweep
        del st
        torch.cuda.empty_cache()
        st = Stack(w, staging, torch, osdp, rows=rows, longer=longer, per_pass=per_pass)

    if not a.no_sweep and a.zdp_slices is None:
        # Section 3.3, last paragraph: the same granularity with fewer and fewer slices in ZDP mode
        zmodes = {}
        kmax = max(max(op.k, 1) for op in w.ops)
        for z in sorted({kmax, kmax // 2, 1, 0}, reverse=True):
            sm = Stack(w, staging, torch, osdp, rows=rows, zdp_slices=z)
            msz = per_step_times(sm, sub_steps, sub_warm, a.serial)[0]
            zmodes[str(z)] = {"tflops": round(flops / (msz * 1e-3) / 1e12, 2), "median_ms_per_step": round(msz, 4),
                              "peak_staging_mb": round(sm.peak_staging / 2 ** 20, 3),
                              "dp_replica_mb": round(sum((max(op.k, 1) - min(z, max(op.k, 1))) * op.I * op.O * 2 / max(op.k, 1)
                                                         for op in w.ops) * w.layers / 2 ** 20, 3)}
            del sm
            torch.cuda.empty_cache()
        out["zdp_slices_of_k"] = zmodes
        out["plan_search"] = plan_search(w, m["kernels"], staging, rows, torch, osdp, sub_steps, sub_warm)
    if not a.no_auto:
        out["auto_granularity"] = auto_granularity(st, osdp, torch, sub_steps, sub_warm)
    if not a.no_sweep and default_plan:
        del st
        torch.cuda.empty_cache()
        out["gemm_8192_cubed_library_vs_vendor"] = library_vs_vendor_gemm(torch, osdp)
        st = Stack(w, staging, torch, osdp, rows=rows, longer=longer, per_pass=per_pass)
    if not a.no_sweep and default_plan:
        # the other workloads under their own plan vectors, each with its own roofline
        also = []
        for cfg in (c for c in (2, 3, 5) if c != a.config):
            del st
            torch.cuda.empty_cache()
            wc = wl.workload(cfg)
            st = Stack(wc, staging, torch, osdp)
            mc = measure(st, wl.flops(wc), sub_steps, sub_warm, False, config=cfg)
            mg = graph_replay_ms(st, sub_steps, sub_warm)
            entry = {"workload": wc.name, "baseline_config": cfg, "plan": {op.name: op.k for op in wc.ops},
                     "graph_replay": {"tflops": round(wl.flops(wc) / (mg * 1e-3) / 1e12, 2), "median_ms_per_step": round(mg, 4)}}
            entry.update({key: mc[key] for key in ("tflops", "frac_bf16_mfma_peak", "median_ms_per_step", "mean_ms_per_step",
                                                   "timed_steps", "peak_staging_mb", "workspace_mb", "roofline", "gathers",
                                                   "idle_us_per_step", "kernels")})
            del st
            torch.cuda.empty_cache()
            st = Stack(wc, staging, torch, osdp, longer=True)
            mlc = per_step_times(st, sub_steps, sub_warm, False)[0]
            entry["longer_split_dim"] = {"tflops": round(wl.flops(wc) / (mlc * 1e-3) / 1e12, 2), "median_ms_per_step": round(mlc, 4),
                                         "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3),
                                         "workspace_mb": round(st.workspace_bytes / 2 ** 20, 3)}
            del st
            torch.cuda.empty_cache()
            st = Stack(wc, staging, torch, osdp, per_pass=True)
            mpc = per_step_times(st, sub_steps, sub_warm, False)[0]
            entry["per_pass_split_dim"] = {"tflops": round(wl.flops(wc) / (mpc * 1e-3) / 1e12, 2), "median_ms_per_step": round(mpc, 4),
                                           "peak_staging_mb": round(st.peak_staging / 2 ** 20, 3),
                                           "workspace_mb": round(st.workspace_bytes / 2 ** 20, 3)}
            also.append(entry)
        out["also"] = also
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, rows=rows)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
