#!/usr/bin/env python3
"""Benchmark of the MuLoCo optimizer hot path on one MI355X.

One "step" is one pass of the whole hot path over a synthetic transformer-shaped parameter
set: a Muon inner step over every 2-D matrix of every resident worker replica (momentum +
look-ahead + norm, batched Newton-Schulz, parameter update), one fused un-quantised outer
step over all groups, and one 4-bit quantised outer step issued as a streaming schedule
would issue it, one layer fragment per call.  All inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

The headline value is the Newton-Schulz matrix-core throughput: FLOP executed by the NS
GEMM launches of the timed steps divided by the summed duration of those launches, each
measured with HIP events on the stream the kernels run on (the library's timing recorder).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = ("Muon step ms + Newton–Schulz TFLOP/s (% MFMA peak); outer step GB/s (% HBM)")
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak


def cpu_baseline(workload, budget_s: float):
    """Time the fp64 oracle (NumPy) on a bounded sample of the workload's matrices."""
    import numpy as np
    import synth_inputs as S
    from oracle import muon
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    d, f = workload.d_model, workload.d_ffn
    shapes = [(min(d, 2048), min(d, 2048)), (min(d, 2048), min(f, 8192))]
    flops = 0.0
    t_used = 0.0
    done = {}
    i = 0
    # alternate over the workload's shapes (capped at 2048 x 8192) until the budget is used
    while t_used < budget_s and i < 64:
        m, n = shapes[i % len(shapes)]
        g = S.normal((m, n), S.GRAD_STD, 0, 999 + i).numpy().astype(np.float64)
        t0 = time.perf_counter()
        muon.newton_schulz(g, 5)
        t_used += time.perf_counter() - t0
        # the oracle always uses the m x m Gram form: 4 m^2 n + 2 m^3 FLOP per iteration
        flops += 5 * (4.0 * m * m * n + 2.0 * m ** 3)
        done[f"{m}x{n}"] = done.get(f"{m}x{n}", 0) + 1
        i += 1
    sample = ", ".join(f"{c} of {k}" for k, c in done.items())
    out = {"value": flops / t_used * 1e-12, "unit": "TFLOP/s", "cores": int(cores),
           "kind": "oracle",
           "sample": "fp64 NumPy Newton-Schulz (5 iterations) on matrices drawn like the workload's: " + sample,
           "seconds": round(t_used, 2)}
    # The elementwise half of the metric: the oracle's outer step (un-quantised, K = 1 and
    # K = 8, and 4-bit quantised at K = 4) on a slice of 1024 rows of one d x f matrix, priced
    # with the same algorithmic bytes per element as the GPU figures.
    from oracle import diloco
    rows, n = 1024, min(f, 8192)
    outer = {}
    for name, K, bits, bpe in (("outer_k1", 1, 0, 4 * 1 + 16), ("outer_k8", 8, 0, 4 * 8 + 16),
                               ("quantised_outer_k4", 4, 4, 4.5 * 4 + 16 + 4 * 4 / n)):
        tg_t = S.normal((rows, n), S.PARAM_STD, 0, 2000)
        tg = tg_t.numpy().astype(np.float64)
        ths = [(tg_t - S.normal((rows, n), S.DELTA_STD, 0, 2001 + k)).to(S.torch_dtype(workload.param_dtype))
               .float().numpy().astype(np.float64) for k in range(K)]
        u0 = np.zeros((rows, n))
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 1.0:
            diloco.outer_step(tg, u0, ths, eta_out=0.9, mu=0.8, quant_bits=bits)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        outer[name] = {"GBps": rows * n * bpe / dt * 1e-9, "ms_per_call": dt * 1e3, "elements": rows * n}
    out["outer_step"] = {"unit": "GB/s of algorithmic bytes", "sample": f"{rows} x {n} slice, fp64 NumPy oracle",
                         **outer}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="1.76b", help="tiny | 150m | 1.76b | 3.1b | 15b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the legs on the 150M- and 3.1B-scale workloads (profiles of one workload's kernels)")
    ap.add_argument("--cpu-budget", type=float, default=12.0)
    ap.add_argument("--workspace-gb", type=float, default=None)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    import synth_inputs as S
    import paper_2505_23725_amd as mlc
    from paper_2505_23725_amd.harness import MulocoJob

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    mlc.library()   # raises if the HIP library is not built
    wl = S.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    cap = None if args.workspace_gb is None else int(args.workspace_gb * 2 ** 30)
    if cap is None and args.workload in ("15b", "3.1b"):
        cap = 8 * 2 ** 30
    job = MulocoJob(wl, device="cuda:0", seed=0, with_quant=True, generate_on="device",
                    workspace_cap_bytes=cap)
    job.draw_gradients(0)
    n_layers = wl.layers

    def step():
        job.inner_step()                       # a1-a6, batched per shape group (a11)
        job.outer_step(0)                      # a7
        hp = job.outer_hparams(quant_bits=4)
        for layer in range(n_layers):          # a8 + a9 as a10: one layer fragment per call
            mlc.muloco_outer_step(job.layer_fragment(layer, quant=True), hp)

    if args.calibration_copy:
        src = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    mlc.muloco_timing_enable(True)
    mlc.muloco_timing_read()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    timing = mlc.muloco_timing_read()
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    # Spread over steps (outside the timed region): the recorder is read after every step, which
    # synchronises, so that each step's Newton-Schulz launches give a figure of their own.
    per_step_tf = []
    for _ in range(args.steps):
        step()
        t1 = mlc.muloco_timing_read()["ns_gemm"]
        if t1["total_ms"] > 0:
            per_step_tf.append(t1["flops"] / (t1["total_ms"] * 1e-3) * 1e-12)
    per_step_tf.sort()
    mlc.muloco_timing_enable(False)

    def spread(v):
        return {"min": v[0], "median": v[len(v) // 2], "max": v[-1]} if v else None

    # Outside the timed region: the stand-alone compressor (codes only), so that it has a
    # figure of its own (inside a step it runs fused with the outer update when rows fit in
    # registers).
    mlc.muloco_timing_enable(True)
    mlc.muloco_timing_read()
    for _ in range(3):
        mlc.muloco_quantize_delta(job.outer_groups(quant=True), job.outer_hparams(quant_bits=4))
    torch.cuda.synchronize()
    extra = mlc.muloco_timing_read()
    mlc.muloco_timing_enable(False)
    q = extra["quantize"]
    quant_alone = {"ms": q["total_ms"] / 3, "GBps": q["bytes"] / (q["total_ms"] * 1e-3) * 1e-9 if q["total_ms"] > 0 else 0.0}
    quant_alone["frac_hbm"] = quant_alone["GBps"] / PEAK_HBM_GBS

    # Also outside the timed region: the quantised outer step over the whole model with error
    # feedback (4 bit), in its 8- and 2-bit forms, in the offset form and with one range per
    # matrix (one more pass over the deltas), when their extra buffers fit in memory.
    variants = {}
    free_bytes = torch.cuda.mem_get_info()[0]
    n_elems = sum(c * m * n for (c, m, n) in job.shapes)
    for name, bits, ef, offset, per_matrix in (("4bit_error_feedback", 4, True, False, False),
                                               ("8bit", 8, False, False, False), ("2bit", 2, False, False, False),
                                               ("4bit_offset_form", 4, False, True, False),
                                               ("4bit_range_per_matrix", 4, False, False, True)):
        need = job.K * n_elems * (bits / 8 + (4 if ef else 0)) + (1 << 30)
        if need > free_bytes:
            variants[name] = None
            continue
        groups = []
        for gi, (c, m, n) in enumerate(job.shapes):
            g = mlc.OuterGroup([job.workers[k][gi] for k in range(job.K)], job.theta_g[gi], job.u[gi])
            g.codes = [torch.empty((c * m, n * bits // 8), dtype=torch.uint8, device="cuda:0") for _ in range(job.K)]
            ranges = c if per_matrix else c * m
            g.scales = [torch.empty((ranges,), dtype=torch.float32, device="cuda:0") for _ in range(job.K)]
            if offset:
                g.offsets = [torch.empty((ranges,), dtype=torch.float32, device="cuda:0") for _ in range(job.K)]
            if ef:
                g.residuals = [torch.zeros((c, m, n), dtype=torch.float32, device="cuda:0") for _ in range(job.K)]
            groups.append(g)
        hpv = job.outer_hparams(quant_bits=bits, error_feedback=ef, ef_beta=0.9)
        hpv.quant_offset, hpv.quant_per_matrix = offset, per_matrix
        mlc.muloco_outer_step(groups, hpv)              # warm-up
        torch.cuda.synchronize()
        mlc.muloco_timing_enable(True)
        mlc.muloco_timing_read()
        for _ in range(2):
            mlc.muloco_outer_step(groups, hpv)
        torch.cuda.synchronize()
        tv = mlc.muloco_timing_read()
        mlc.muloco_timing_enable(False)
        ms = sum(tv[k]["total_ms"] for k in ("quantize", "dequant_outer"))
        nbytes = sum(tv[k]["bytes"] for k in ("quantize", "dequant_outer"))
        gbs = nbytes / (ms * 1e-3) * 1e-9 if ms > 0 else 0.0
        variants[name] = {"ms": ms / 2, "GBps": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        del groups
        torch.cuda.empty_cache()

    # Top-k sparsified outer step (5 % kept, error feedback) over the whole model: three selection
    # passes and the sparsified update.
    topk_fig = None
    if job.K * n_elems * 4 + (1 << 30) < torch.cuda.mem_get_info()[0]:
        groups = []
        for gi, (c, m, n) in enumerate(job.shapes):
            g = mlc.OuterGroup([job.workers[k][gi] for k in range(job.K)], job.theta_g[gi], job.u[gi])
            g.residuals = [torch.zeros((c, m, n), dtype=torch.float32, device="cuda:0") for _ in range(job.K)]
            groups.append(g)
        hpt = job.outer_hparams(error_feedback=True, ef_beta=0.9)
        wsp = torch.empty(mlc.muloco_topk_workspace_bytes(groups, job.K), dtype=torch.uint8, device="cuda:0")
        mlc.muloco_topk_outer_step(groups, hpt, 0.05, wsp)
        torch.cuda.synchronize()
        mlc.muloco_timing_enable(True)
        mlc.muloco_timing_read()
        for _ in range(2):
            mlc.muloco_topk_outer_step(groups, hpt, 0.05, wsp)
        torch.cuda.synchronize()
        tt = mlc.muloco_timing_read()["topk"]
        mlc.muloco_timing_enable(False)
        gbs = tt["bytes"] / (tt["total_ms"] * 1e-3) * 1e-9 if tt["total_ms"] > 0 else 0.0
        # the method's own bytes: one read of theta_k, E_k, theta_g and u and one write of E_k,
        # theta_g, u and theta_k; the three selection passes are this implementation's cost
        method_bytes = n_elems * (12 * job.K + 16)
        mgbs = method_bytes / (tt["total_ms"] / 2 * 1e-3) * 1e-9 if tt["total_ms"] > 0 else 0.0
        topk_fig = {"ms": tt["total_ms"] / 2, "passes": 4,
                    "executed_bytes_GBps": gbs, "executed_bytes_frac_hbm": gbs / PEAK_HBM_GBS,
                    "algorithmic_bytes_GBps": mgbs, "algorithmic_bytes_frac_hbm": mgbs / PEAK_HBM_GBS}
        del groups, wsp
        torch.cuda.empty_cache()

    # AdamW on a tensor the size of an embedding plus an output layer (2 x 32768 x d_model), the
    # kind of parameter Muon does not cover; outside the timed region.
    adamw_fig = None
    n_emb = 2 * 32768 * wl.d_model
    if 24 * n_emb + (1 << 30) < torch.cuda.mem_get_info()[0]:
        pdt = S.torch_dtype(wl.param_dtype)
        emb = S.normal((n_emb,), S.PARAM_STD, 0, 77, device="cuda:0", dtype=pdt)
        gemb = S.normal((n_emb,), S.GRAD_STD, 0, 78, device="cuda:0", dtype=pdt)
        m1 = torch.zeros(n_emb, dtype=torch.float32, device="cuda:0")
        m2 = torch.zeros(n_emb, dtype=torch.float32, device="cuda:0")
        hpa = mlc.AdamWHParams(lr=1e-3, weight_decay=0.1, bias_correction=True, step=1)
        mlc.muloco_adamw_step([(emb, gemb, m1, m2)], hpa)
        torch.cuda.synchronize()
        mlc.muloco_timing_enable(True)
        mlc.muloco_timing_read()
        for i in range(3):
            hpa.step = 2 + i
            mlc.muloco_adamw_step([(emb, gemb, m1, m2)], hpa)
        torch.cuda.synchronize()
        ta = mlc.muloco_timing_read()["adamw"]
        mlc.muloco_timing_enable(False)
        gbs = ta["bytes"] / (ta["total_ms"] * 1e-3) * 1e-9 if ta["total_ms"] > 0 else 0.0
        adamw_fig = {"elements": n_emb, "ms": ta["total_ms"] / 3, "GBps": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        del emb, gemb, m1, m2
        torch.cuda.empty_cache()

    # The same step replayed from a HIP graph (one submission per step instead of one per
    # kernel): what launch overhead costs on the small workloads.
    graph_ms = None
    try:
        graph = MulocoJob.capture(step)
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg0) * 1e3 / args.steps
        del graph
    except Exception as e:          # the eager figures stand without it
        graph_ms = f"failed: {e}"

    # Workloads whose whole state fits the caches (L2 and the 256 MB memory-side cache): the same
    # step with the caches flushed before each one (a 1 GiB fill), timed step by step.
    flushed_ms = None
    state_bytes = n_elems * job.K * 16
    if state_bytes < (256 << 20):
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        per = []
        for i in range(max(3, args.steps)):
            flush.fill_(i & 0xff)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            step()
            e1.record()
            torch.cuda.synchronize()
            per.append(e0.elapsed_time(e1))
        per.sort()
        flushed_ms = {"min": per[0], "median": per[len(per) // 2], "max": per[-1]}
        del flush
        torch.cuda.empty_cache()

    # The outer-step half of the metric on the configurations it is quoted on (outside the timed
    # region, outer state only): the fused un-quantised step on the 150M-scale set with K = 8
    # replicas, and the 4-bit quantised step on the 3.1B-scale shapes with K = 4.
    n_elems_main, K_main = n_elems, job.K
    nominal = job.ns_flops() * job.K
    del job
    torch.cuda.empty_cache()

    def outer_on(workload_name, quant_bits, reps):
        w2 = S.WORKLOADS[workload_name]
        need = w2.n_params() * (2 * w2.K + 8 + (w2.K * quant_bits / 8 if quant_bits else 0)) + (4 << 30)
        if need > torch.cuda.mem_get_info()[0]:
            return None
        j2 = MulocoJob(w2, device="cuda:0", seed=0, with_quant=quant_bits != 0, generate_on="device",
                       outer_only=True)
        j2.displace_workers()
        hp2 = j2.outer_hparams(quant_bits=quant_bits)
        groups = j2.outer_groups(quant=quant_bits != 0)
        fam_name = "dequant_outer" if quant_bits else "outer"
        mlc.muloco_outer_step(groups, hp2)
        torch.cuda.synchronize()
        mlc.muloco_timing_enable(True)
        mlc.muloco_timing_read()
        per_call = []
        tot_ms = tot_bytes = 0.0
        for _ in range(reps):
            mlc.muloco_outer_step(groups, hp2)
            t2 = mlc.muloco_timing_read()[fam_name]
            per_call.append(t2["total_ms"])
            tot_ms += t2["total_ms"]
            tot_bytes += t2["bytes"]
        fig = {"workload": f"{w2.name}-scale, K={w2.K}, {w2.n_params()} elements per replica",
               "ms": tot_ms / reps, "ms_min": min(per_call), "ms_median": sorted(per_call)[reps // 2],
               "bytes_per_element": tot_bytes / reps / w2.n_params(),
               "GBps": tot_bytes / (tot_ms * 1e-3) * 1e-9, "frac_hbm": tot_bytes / (tot_ms * 1e-3) * 1e-9 / PEAK_HBM_GBS}
        if quant_bits:      # the compressor alone (codes and scales only)
            mlc.muloco_quantize_delta(groups, hp2)
            torch.cuda.synchronize()
            mlc.muloco_timing_read()
            for _ in range(reps):
                mlc.muloco_quantize_delta(groups, hp2)
            tq = mlc.muloco_timing_read()["quantize"]
            qg = tq["bytes"] / (tq["total_ms"] * 1e-3) * 1e-9 if tq["total_ms"] > 0 else 0.0
            fig["quantiser_alone"] = {"ms": tq["total_ms"] / reps, "GBps": qg, "frac_hbm": qg / PEAK_HBM_GBS}
        mlc.muloco_timing_enable(False)
        del j2, groups
        torch.cuda.empty_cache()
        return fig

    def inner_on(workload_name, reps):
        """Muon inner step of another workload (all its replicas), outside the timed region."""
        w2 = S.WORKLOADS[workload_name]
        j2 = MulocoJob(w2, device="cuda:0", seed=0, generate_on="device")
        j2.draw_gradients(0)
        for _ in range(2):
            j2.inner_step()
        torch.cuda.synchronize()
        mlc.muloco_timing_enable(True)
        mlc.muloco_timing_read()
        per = []
        tot = {"ms": 0.0, "flops": 0.0, "launches": 0, "all_ms": 0.0}
        for _ in range(reps):
            j2.inner_step()
            t2 = mlc.muloco_timing_read()
            g2 = t2["ns_gemm"]
            per.append(g2["flops"] / (g2["total_ms"] * 1e-3) * 1e-12 if g2["total_ms"] > 0 else 0.0)
            tot["ms"] += g2["total_ms"]; tot["flops"] += g2["flops"]; tot["launches"] += g2["launches"]
            tot["all_ms"] += sum(t2[k]["total_ms"] for k in ("ns_gemm", "momentum", "norm", "update"))
        mlc.muloco_timing_enable(False)
        tf = tot["flops"] / (tot["ms"] * 1e-3) * 1e-12 if tot["ms"] > 0 else 0.0
        fig = {"workload": f"{w2.name}-scale, K={w2.K}", "muon_inner_step_ms": tot["all_ms"] / reps,
               "ns_gemm_ms": tot["ms"] / reps, "ns_gemm_launches": tot["launches"] / reps,
               "ns_tflops": tf, "frac_mfma": tf / PEAK_BF16_TFLOPS, "ns_tflops_spread": spread(sorted(per))}
        del j2
        torch.cuda.empty_cache()
        return fig

    others = not args.no_other_workloads
    ns_150m = inner_on("150m", 10) if others and wl.name != "150m" else None
    outer_k8_150m = outer_on("150m", 0, 10) if others else None
    quantised_outer_k4_31b = outer_on("3.1b", 4, 3) if others else None

    ms_per_step = wall * 1e3 / args.steps
    gemm = timing["ns_gemm"]
    ns_tflops = gemm["flops"] / (gemm["total_ms"] * 1e-3) * 1e-12 if gemm["total_ms"] > 0 else 0.0

    def fam(name):
        t = timing[name]
        gbs = t["bytes"] / (t["total_ms"] * 1e-3) * 1e-9 if t["total_ms"] > 0 else 0.0
        out = {"ms_per_step": t["total_ms"] / args.steps, "launches_per_step": t["launches"] / args.steps,
               "GBps": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        if name == "update" and t["launches"] == 0:
            out = {"ms_per_step": 0.0, "launches_per_step": 0.0,
                   "note": "bf16 weights: the update is the epilogue of the last Newton-Schulz product"}
        return out

    inner_ms = sum(timing[k]["total_ms"] for k in ("ns_gemm", "momentum", "norm", "update")) / args.steps
    breakdown = {
        "muon_inner_step_ms": inner_ms,
        "ns_gemm_ms_per_step": gemm["total_ms"] / args.steps,
        "ns_gemm_launches_per_step": gemm["launches"] / args.steps,
        "ns_flop_per_step": gemm["flops"] / args.steps,
        "momentum": fam("momentum"), "update": fam("update"), "outer": fam("outer"),
        "quantize_outer_fused": fam("dequant_outer"),
        "ns_150m_k8": ns_150m,
        "outer_k8_150m": outer_k8_150m,
        "quantised_outer_k4_3.1b": quantised_outer_k4_31b,
        "step_ms_spread": spread(step_ms),
        "ns_tflops_per_step_spread": spread(per_step_tf),
        "graph_replay_ms_per_step": graph_ms,
        "flushed_cache_ms_per_step": flushed_ms,
        "adamw_embedding_sized_tensor": adamw_fig,
        "topk_5pct_error_feedback_outer_step_whole_model": topk_fig,
        "quantize_standalone_whole_model": quant_alone,
        "quantised_outer_step_whole_model_variants": variants,
        "nominal_ns_tflops_equivalent": None,
    }
    breakdown["nominal_ns_tflops_equivalent"] = nominal / (gemm["total_ms"] / args.steps * 1e-3) * 1e-12 if gemm["total_ms"] > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"ns_gemm_bf16_kernel_{wl.name}_traffic.txt")
    if os.path.exists(tpath):       # HBM bytes per launch from the rocprofv3 --pmc runs
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split()[1])
    out = {
        "metric": METRIC,
        "value": ns_tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}-scale: {wl.layers} layers, d_model {wl.d_model}, FFN {wl.d_ffn}, "
                               f"K={K_main} replicas, {wl.param_dtype} params, fp32 momentum",
                   "params_2d": wl.n_params(), "ns_iters": 5,
                   "step": "muon inner step + fused outer step + 4-bit quantised outer step per layer fragment"},
        "roofline": {"bound": "mfma", "achieved": ns_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": ns_tflops / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": (None if traffic is None else
                                        f"profiles/ns_gemm_bf16_kernel_{wl.name}_traffic.txt (rocprofv3 --pmc runs of this "
                                        "command; read from the file, not measured in this run)"),
                     # shapes of at most 128 x 512 run the whole chain in one launch instead
                     "kernel": ("ns_chain_small_kernel" if max(wl.d_model, wl.d_ffn) <= 512 and wl.d_model <= 128
                                else "ns_gemm_bf16_kernel"),
                     "avg_launch_ms": gemm["total_ms"] / max(1, gemm["launches"])},
        "breakdown": breakdown,
    }
    # Achievable peaks of this chip from the microbenchmark executable (a child process).
    try:
        import subprocess
        from paper_2505_23725_amd.build import MICROBENCH_PATH
        res = subprocess.run([MICROBENCH_PATH], capture_output=True, text=True, timeout=120)
        out["achievable"] = json.loads(res.stdout.strip().splitlines()[-1])
        # operands drawn like the workload's; the random-bit-pattern figure is the worst case
        ach = out["achievable"]["mfma_bf16_tflops_gaussian_operands"]
        out["roofline"]["frac_of_achievable"] = ns_tflops / ach if ach > 0 else None
        # every GB/s figure also against what a plain in-place read-modify-write stream reaches
        # on this machine (all of the elementwise kernels are such streams)
        rmw = out["achievable"].get("hbm_rmw_in_place_GBps", 0)

        def annotate(d):
            if isinstance(d, dict):
                if rmw and isinstance(d.get("GBps"), (int, float)):
                    d["frac_of_measured_rmw_stream"] = d["GBps"] / rmw
                for v in list(d.values()):
                    annotate(v)
        annotate(breakdown)
    except Exception as e:      # the benchmark stands without it
        out["achievable"] = {"error": str(e)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_budget)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
