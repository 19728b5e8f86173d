#!/usr/bin/env python3
"""Throughput of the MI355X Muon step on the synthetic LLM-shaped matrix sets.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--no-cpu-baseline]

One "step" is one muon_step over the whole matrix list of the workload: momentum, Frobenius norm,
cast/orient, N Newton-Schulz iterations (three grouped GEMMs each) and the scaled weight-decayed update.
Inputs are generated on the device before the timed region.  Prints ONE JSON line.

The roofline object describes the dominant kernel (the bf16 MFMA GEMM of the Newton-Schulz products):
nominal flops per launch = N*(4 m^2 n + 2 m^3) summed over matrices / launches per step, divided by the
average launch duration measured with HIP events on the step's stream inside the timed region.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_F32_VALU_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
DEFAULT_CONFIG = "block_w4096"
# every single-GPU workload of the target: (name, timed steps, warm-up steps) when it is not the headline
OTHER_WORKLOADS = (("block_w4096", 5, 2), ("dense12_w1024", 5, 2), ("moe_bank_66x2048x1408", 5, 2), ("moe27_w2048", 3, 1))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload, ns_dtype):
    """HBM-side bytes per launch of the dominant kernel, from profiles/traffic.json: rocprofv3 FETCH_SIZE /
    WRITE_SIZE runs of this same script (commands and commit recorded there), scaled by the counters' reading for a
    plain copy (--calibrate-copy).  Not measured by this run; None when no profile covers the workload."""
    try:
        with open(TRAFFIC_FILE) as f:
            entry = json.load(f)["workloads"].get(f"{workload}:{ns_dtype}")
    except (OSError, ValueError, KeyError):
        return None, None
    if not entry:
        return None, None
    return int(entry["bytes_per_launch"]), f"profiles/traffic.json ({entry.get('measured_at', 'unknown commit')}), not this run"


def calibrate_copy(mib=1024, repeats=5):
    """Plain device-to-device copies of a known size, for calibrating rocprofv3's FETCH_SIZE / WRITE_SIZE counters:
    each repeat is one torch copy kernel that reads and writes exactly `mib` MiB."""
    import torch
    n = mib * 2 ** 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(repeats):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes": n, "repeats": repeats}), flush=True)
    return 0


def executed_ns_flops(wl, ns_steps, ns_dtype="bf16"):
    """Matrix-core flops actually issued, summed over the tile tables of the launch plan (host-only call into the
    library): symmetric products compute only tiles on or above the diagonal and, in plain bf16, only the upper triangle
    of 32 x 32 blocks of a diagonal tile; strip tiles that were shifted to end at the matrix edge recompute what they
    overlap."""
    from paper_2502_16982_amd import binding
    n = len(wl.shapes)
    p = binding.param_array(wl.shapes, [1] * n, [1] * n)
    ns = binding.NS_DTYPES[ns_dtype]
    ctx = binding.muon_plan_only(p, n, ns, binding.muon_workspace_bytes(p, n, ns, 0))
    try:
        desc = [binding.muon_plan_describe(ctx, i) for i in range(n)]
        flops = 0
        for product, k_of in (("gram", "n_pad"), ("poly", "m_pad"), ("apply", "m_pad")):
            for level in (0, 1):
                for mat, _, _, _, _, blocks in binding.muon_plan_tiles(ctx, 0, product, level):
                    flops += 2 * blocks * 1024 * desc[mat][k_of]
    finally:
        binding.muon_destroy(ctx)
    return ns_steps * flops


def cpu_baseline(wl, budget_s=25.0):
    """Times the fp64 oracle (as it stands) on the host cores on a bounded sample of the workload."""
    import numpy as np
    import torch
    from oracle import muon_oracle as orc
    from paper_2502_16982_amd import workloads
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    h = wl.hyper
    # one matrix per distinct shape, cheapest first, until the budget is used
    seen = {}
    for i, s in enumerate(wl.shapes):
        seen.setdefault(s, i)
    order = sorted(seen.items(), key=lambda kv: min(kv[0]) ** 2 * max(kv[0]))
    flops_done, t_done, sample = 0, 0.0, []
    for shape, idx in order:
        m, n = min(shape), max(shape)
        fl = h.ns_steps * (4 * m * m * n + 2 * m ** 3)
        if sample and t_done > 0 and t_done + fl * (t_done / flops_done) > budget_s:
            continue
        w, g, mom = workloads.make_matrix(wl, idx, "cpu")
        w64, g64, m64 = (t.float().numpy().astype(np.float64) for t in (w, g, mom))
        t0 = time.perf_counter()
        orc.muon_step(w64, g64, m64, lr=h.lr, weight_decay=h.weight_decay, mu=h.momentum, ns_steps=h.ns_steps,
                      eps=h.eps, nesterov=h.nesterov)
        dt = time.perf_counter() - t0
        flops_done += fl
        t_done += dt
        sample.append(f"{shape[0]}x{shape[1]}:{dt:.2f}s")
    total = wl.ns_flops()
    est_step_s = t_done * total / flops_done
    return {"value": 1.0 / est_step_s, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": "fp64 numpy oracle, one full step on one matrix per sampled shape (" + ", ".join(sample) +
                      f"), scaled to the whole list by nominal NS flops ({flops_done:.3e} of {total:.3e})",
            "gflops": flops_done / t_done / 1e9}


def bench_adamw(dev, steps=5):
    """HBM rate of the AdamW kernel on the non-matrix parameters of a width-2048 model (embedding and LM head of
    163840 x 2048 bf16, 55 RMSNorm gains), timed with events on the launch stream."""
    import torch
    from paper_2502_16982_amd import binding
    sizes = [163840 * 2048, 163840 * 2048] + [2048] * 55
    tensors = []
    for n in sizes:
        tensors.append((torch.empty(n, dtype=torch.bfloat16, device=dev).normal_(0, 0.02),
                        torch.empty(n, dtype=torch.bfloat16, device=dev).normal_(0, 1e-3),
                        torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=torch.float32, device=dev)))
    stream = torch.cuda.current_stream(dev)
    binding.muon_adamw_step(tensors, lr=4.2e-4, weight_decay=0.1, step=1, stream_ptr=stream.cuda_stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for t in range(steps):
        binding.muon_adamw_step(tensors, lr=4.2e-4, weight_decay=0.1, step=2 + t, stream_ptr=stream.cuda_stream)
    e1.record(stream)
    e1.synchronize()
    ms = e0.elapsed_time(e1) / steps
    n_el = sum(sizes)
    gbs = n_el * 22 / (ms * 1e-3) / 1e9      # p 2+2, g 2, m 4+4, v 4+4 bytes per element
    return {"elements": n_el, "ms_per_step": ms, "algorithmic_GBs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}


PLANES = {"f32": 1, "bf16": 1, "bf16x2": 2, "bf16x3": 3}     # bf16 arrays per Newton-Schulz temporary
SEGMENTS = {1: 1, 2: 3, 3: 6}                                 # matrix-core products behind one product of Eq. 2


def time_workload(name, steps, warmup, max_ws_gib, dev, ns_dtype=None):
    """W untimed warm-up steps, then exactly `steps` timed steps of the whole hot path over workload `name`
    (inputs generated on the device beforehand), bracketed by device synchronisation.  Per-kernel-class times come
    from HIP events the library records around every launch on the step's stream inside the timed region."""
    import torch
    from paper_2502_16982_amd import binding, workloads
    wl = workloads.workload(name)
    if ns_dtype is not None:
        wl = dataclasses.replace(wl, ns_dtype=ns_dtype)
    h = wl.hyper
    tensors = workloads.make_all(wl, dev)
    st = binding.MuonStepper(tensors, ns_dtype=wl.ns_dtype, max_workspace_bytes=int(max_ws_gib * 2 ** 30))
    hp = binding.default_hparams(lr=h.lr, weight_decay=h.weight_decay, momentum=h.momentum, eps=h.eps,
                                 ns_steps=h.ns_steps, nesterov=int(h.nesterov))
    stream = torch.cuda.current_stream(dev)

    for _ in range(warmup):
        st.step(hp, stream=stream)
    torch.cuda.synchronize()
    binding.muon_profile_enable(st.ctx, True)
    binding.muon_profile_read(st.ctx, reset=True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        st.step(hp, stream=stream)
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    prof = binding.muon_profile_read(st.ctx, reset=True)
    binding.muon_profile_enable(st.ctx, False)

    ms_per_step = elapsed * 1e3 / steps
    nominal = wl.ns_flops()
    gemm_ms = sum(prof[k][0] for k in ("gram", "poly", "apply_poly"))
    gemm_launches = sum(prof[k][1] for k in ("gram", "poly", "apply_poly"))
    bf16 = wl.ns_dtype != "f32"              # the matrix-core paths: plain bf16 and the split forms
    planes = PLANES[wl.ns_dtype]
    executed = executed_ns_flops(wl, h.ns_steps, wl.ns_dtype) * SEGMENTS[planes]
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_VALU_TFLOPS
    if gemm_launches:
        avg_launch_ms = gemm_ms / gemm_launches
        flops_per_launch = nominal * steps / gemm_launches
        achieved = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12
    else:
        avg_launch_ms, flops_per_launch, achieved = 0.0, 0.0, 0.0
    traffic, traffic_source = measured_traffic(wl.name, wl.ns_dtype)
    roofline = {"bound": "mfma" if bf16 else "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                "frac": achieved / peak, "traffic": traffic, "traffic_source": traffic_source,
                "kernel": "ns_gemm_bf16_kernel" if bf16 else "ns_gemm_f32_kernel",
                "avg_launch_ms": avg_launch_ms, "launches_per_step": gemm_launches / max(steps, 1),
                "nominal_flops_per_launch": flops_per_launch,
                "executed_tflops": executed * steps / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0,
                "executed_frac": executed * steps / (gemm_ms * 1e-3) / 1e12 / peak if gemm_ms else 0.0}

    n_el = wl.n_elements
    g_b = 2 if wl.g_dtype == torch.bfloat16 else 4
    w_b = 2 if wl.w_dtype == torch.bfloat16 else 4
    x_b = 2 * planes if bf16 else 4
    ew = {}
    for key, bytes_per_el in (("momentum_norm_cast", g_b + 8 + x_b), ("weight_update", 2 * w_b + x_b)):
        ms, cnt = prof[key]
        if cnt:
            ew[key] = {"ms_per_step": ms / steps, "algorithmic_GBs": n_el * bytes_per_el * steps / (ms * 1e-3) / 1e9,
                       "frac_of_hbm_peak": n_el * bytes_per_el * steps / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    chunks, ws_bytes = binding.muon_plan_chunks(st.ctx), st.workspace_bytes
    st.close()
    del tensors
    torch.cuda.empty_cache()
    return {"wl": wl, "hyper": h, "bf16": bf16, "planes": planes, "steps": steps, "elapsed": elapsed, "ms_per_step": ms_per_step,
            "nominal": nominal,
            "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
            "executed": executed, "gemm_ms": gemm_ms, "prof": prof, "roofline": roofline, "elementwise": ew, "n_el": n_el,
            "chunks": chunks, "workspace_bytes": ws_bytes}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="time only --config, not the other workloads as well")
    ap.add_argument("--max-workspace-gib", type=float, default=16.0)
    ap.add_argument("--ns-dtype", choices=sorted(PLANES), default=None,
                    help="Newton-Schulz arithmetic of --config (default: the workload's own, bf16 for the headline)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run five plain 1 GiB device copies (counter calibration under rocprofv3 --pmc) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2502_16982_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.lib()
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        return calibrate_copy()
    r = time_workload(args.config, args.steps, args.warmup, args.max_workspace_gib, dev, args.ns_dtype)
    wl, h, bf16 = r["wl"], r["hyper"], r["bf16"]
    elapsed, ms_per_step, nominal, executed = r["elapsed"], r["ms_per_step"], r["nominal"], r["executed"]
    gemm_ms, prof, roofline, ew, n_el = r["gemm_ms"], r["prof"], r["roofline"], r["elementwise"], r["n_el"]

    out = {
        "metric": "muon_steps_per_sec", "value": args.steps / elapsed, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.ns_dtype, "data": "synthetic",
        "config": {"workload": wl.name, "matrices": len(wl.shapes), "elements": n_el,
                   "w_dtype": str(wl.w_dtype).replace("torch.", ""), "g_dtype": str(wl.g_dtype).replace("torch.", ""),
                   "momentum_dtype": "float32", "ns_steps": h.ns_steps, "nesterov": bool(h.nesterov),
                   "chunks": r["chunks"], "workspace_bytes": r["workspace_bytes"]},
        "ns_tflops_whole_step": nominal / (ms_per_step * 1e-3) / 1e12,
        "ns_tflops_gemm_time": nominal * args.steps / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
        "ns_pct_of_bf16_peak_whole_step": 100.0 * nominal / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "nominal_ns_flops_per_step": nominal, "executed_ns_flops_per_step": executed,
        "kernel_ms_per_step": {k: v[0] / args.steps for k, v in prof.items() if v[1]},
        "elementwise": ew,
        "roofline": roofline,
    }
    if not args.no_others:
        # The other single-GPU workloads of the target, each through the same timed loop (fewer steps); the headline
        # fields above stay those of --config.
        out["other_workloads"] = []
        for other, o_steps, o_warm in OTHER_WORKLOADS:
            if other == args.config:
                continue
            o = time_workload(other, o_steps, o_warm, args.max_workspace_gib, dev)
            out["other_workloads"].append({
                "workload": other, "steps": o_steps, "warmup": o_warm, "matrices": len(o["wl"].shapes), "elements": o["n_el"],
                "chunks": o["chunks"], "workspace_bytes": o["workspace_bytes"],
                "ms_per_step": o["ms_per_step"], "steps_per_s": 1e3 / o["ms_per_step"],
                "ms_per_step_median": o["ms_per_step_median"], "ms_per_step_min": o["ms_per_step_min"],
                "ns_tflops_whole_step": o["nominal"] / (o["ms_per_step"] * 1e-3) / 1e12,
                "ns_gemm_tflops_nominal": o["roofline"]["achieved"], "frac_of_bf16_peak": o["roofline"]["frac"],
                "ns_gemm_tflops_executed": o["roofline"]["executed_tflops"],
                "avg_gemm_launch_ms": o["roofline"]["avg_launch_ms"], "launches_per_step": o["roofline"]["launches_per_step"],
                "roofline": o["roofline"],
                "kernel_ms_per_step": {k: v[0] / o_steps for k, v in o["prof"].items() if v[1]},
                "elementwise": o["elementwise"]})
        if args.ns_dtype is None:
            # the accurate matrix-core path on the headline workload: two bf16 planes, three products per product of Eq. 2
            o = time_workload(args.config, min(5, max(2, args.steps // 2)), 2, args.max_workspace_gib, dev, "bf16x2")
            out["accurate_path"] = {
                "workload": args.config, "ns_dtype": "bf16x2", "ms_per_step": o["ms_per_step"],
                "ms_per_step_median": o["ms_per_step_median"], "steps_per_s": 1e3 / o["ms_per_step"],
                "ns_gemm_tflops_nominal": o["roofline"]["achieved"],
                "matrix_core_tflops_executed": o["roofline"]["executed_tflops"],
                "avg_gemm_launch_ms": o["roofline"]["avg_launch_ms"], "roofline": o["roofline"],
                "kernel_ms_per_step": {k: v[0] / o["steps"] for k, v in o["prof"].items() if v[1]},
                "elementwise": o["elementwise"], "workspace_bytes": o["workspace_bytes"], "chunks": o["chunks"]}
    out["adamw_non_matrix_params"] = bench_adamw(dev)
    torch.cuda.empty_cache()
    if bf16:
        # Context for roofline.frac (which stays priced against the published peak): what the matrix cores sustain
        # on register-resident operands right now, on this chip, with random and with all-zero operand values.
        rnd = binding.muon_probe_mfma_rate(True)
        zer = binding.muon_probe_mfma_rate(False)
        out["roofline"]["mfma_register_loop"] = {
            "random_operands_tflops": rnd["tflops"], "random_operands_clock_mhz": rnd["clock_mhz"],
            "zero_operands_tflops": zer["tflops"], "zero_operands_clock_mhz": zer["clock_mhz"],
            "executed_frac_of_random_operand_rate": (out["roofline"]["executed_tflops"] / rnd["tflops"]) if rnd["tflops"] else None,
            "nominal_frac_of_random_operand_rate": (out["roofline"]["achieved"] / rnd["tflops"]) if rnd["tflops"] else None}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
