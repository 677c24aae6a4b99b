#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one pass of the whole path over one batch of seeded synthetic input
already resident in HBM: gate, slot assignment, and per partition dispatch,
expert FFN forward, combine, then the backward pass (moe_layer_step).  Prints one
JSON line with the whole-step throughput, the roofline of the dominant kernel
(the bf16 MFMA grouped GEMM) measured with HIP events inside the timed region,
the HBM-bound permutation kernels beside it, workspace bytes per memory-reuse
mode, and the CPU oracle timed on a bounded sample of the same workload.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large] [--n 2] [--reuse 2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

GEMM_KINDS = ("gemm_fwd1_gelu", "gemm_nn_store", "gemm_dgelu", "gemm_dgrad", "gemm_wgrad")


def cpu_baseline(shape, inp, budget_tokens):
    """The oracle as it stands, timed on a token slice of the same workload."""
    import numpy as np
    from oracle import moe_oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ts = min(shape.T, budget_tokens)
    t0 = time.perf_counter()
    moe_oracle.layer_step(inp["x"][:Ts], inp["Wg"], inp["W1"], inp["W2"], inp["dy"][:Ts], shape.k,
                          shape.capacity_factor, 1, gate_bias=inp.get("gate_bias"))
    dt = time.perf_counter() - t0
    return {"value": Ts / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {Ts} of {shape.T} tokens, full weights, one partition, float64 numpy, {dt:.1f} s"}


def recorded_traffic(workload, n, reuse):
    """HBM-side bytes per GEMM launch recorded from rocprofv3 --pmc runs (FETCH_SIZE +
    WRITE_SIZE, calibrated on the dispatch kernel) and where the record is; (None, None) if
    there is none for this setup.  A recorded value, not a measurement of this run: counters
    need runs of their own."""
    name = f"hbm_traffic_{workload}_n{n}_reuse{reuse}.txt"
    path = os.path.join(ROOT, "profiles", name)
    try:
        val, date = None, "undated"
        for line in open(path):
            if line.startswith("gemm_traffic_bytes_per_launch"):
                val = float(line.split()[1])
            if line.startswith("recorded "):
                date = line.split(None, 1)[1].strip()
        if val is not None:
            return val, f"recorded by rocprofv3 --pmc, profiles/{name} ({date}); not measured in this run"
    except OSError:
        pass
    return None, None


def measure(args, workload, n, reuse, steps, warmup, brief=False, fuse=0, group=0):
    """Time `steps` whole layer steps of one workload; returns the result dict and the inputs."""
    import numpy as np
    import torch
    from paper_2506_22175_amd import binding as B
    from paper_2506_22175_amd import runner, synth

    shape = synth.WORKLOADS[workload]
    inp = synth.make_inputs(shape, seed=0)
    st = runner.LayerState(shape.T, shape.M, shape.H, shape.E, shape.k, shape.capacity_factor, n,
                           shape.dtype, reuse, second_stream=not args.single_stream,
                           grad_overwrite=0 if args.accumulate else 1, fuse_gather=fuse, wgrad_group=group)
    st.upload(inp)
    st.zero_grads()
    torch.cuda.reset_peak_memory_stats()

    for _ in range(warmup):
        st.step()
    torch.cuda.synchronize()

    graph = st.capture() if args.graph else None
    run_step = graph.replay if graph is not None else st.step
    if graph is not None:
        for _ in range(2):
            run_step()
    B.moe_profile_enable(graph is None and not args.no_kernel_timing)
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(st.s0)
    for _ in range(steps):
        run_step()
    ev1.record(st.s0)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    B.moe_profile_enable(False)
    prof = B.moe_profile_read()
    kernel_timing = "HIP events on each kernel's own stream, inside the timed region"
    if graph is not None:
        # a graph replay cannot carry the timing events: time the kernels in an eager pass after it
        B.moe_profile_enable(True)
        for _ in range(steps):
            st.step()
        torch.cuda.synchronize()
        B.moe_profile_enable(False)
        prof = B.moe_profile_read()
        kernel_timing = "HIP events in an eager pass of the same number of steps after the timed graph replays"
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall_ms / steps
    peak_alloc = torch.cuda.max_memory_allocated()
    ws_bytes = int(st.ws_total)

    counts = st.counts.cpu().numpy()
    slot = st.slot.cpu().numpy()
    R = int(counts.sum())                       # kept rows over all partitions
    drop_rate = float((slot < 0).mean())
    T, M, H, k = shape.T, shape.M, shape.H, shape.k
    es = 2 if shape.dtype == "bf16" else 4
    gemms_per_row = {"gemm_fwd1_gelu": 1, "gemm_nn_store": 1 + (1 if reuse == 2 else 0), "gemm_dgelu": 1,
                     "gemm_dgrad": 1, "gemm_wgrad": 2}
    flop_model = 12.0 * R * M * H
    flop_exec = flop_model + (2.0 * R * M * H if reuse == 2 else 0.0)

    # dominant kernel: the grouped GEMM (all five uses of the one MFMA kernel)
    g_launch = sum(prof[kd][0] for kd in GEMM_KINDS)
    g_ms = sum(prof[kd][1] for kd in GEMM_KINDS)
    g_flop_per_step = sum(2.0 * R * M * H * gemms_per_row[kd] for kd in GEMM_KINDS)
    achieved_tflops = g_flop_per_step * steps / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    per_kind = {}
    for kd in GEMM_KINDS:
        l, ms = prof[kd]
        if l:
            per_kind[kd] = {"launches": l, "avg_us": 1e3 * ms / l,
                            "tflops": 2.0 * R * M * H * gemms_per_row[kd] * steps / (ms * 1e-3) / 1e12}
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_kernel (grouped expert GEMM, all layouts)",
                "achieved": achieved_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved_tflops / PEAK_BF16_TFLOPS,
                "traffic": recorded_traffic(workload, n, reuse)[0] if not group else None,
                "traffic_source": recorded_traffic(workload, n, reuse)[1] if not group else None,
                "launches": g_launch, "avg_launch_us": 1e3 * g_ms / max(g_launch, 1),
                "flop_per_launch": g_flop_per_step * steps / max(g_launch, 1), "per_use": per_kind,
                "kernel_timing": kernel_timing}

    # HBM-bound permutations: algorithmic bytes = rows read + rows written
    # x forward (not with the gathered first GEMM); dy backward, and x again when T_DI is not where forward left it
    n_disp_per_step = (0 if fuse else 1) + (2 if (fuse or (reuse in (1, 2, 4) and n > 2)) else 1)
    # dispatch reads every token row once, however many experts it goes to, and writes the kept rows
    # (counting a read per kept row, 2*R rows, would flatter the kernel by a quarter at k = 2)
    bytes_dispatch = (R + T) * M * es + T * k * 4.0         # per dispatch of all partitions
    bytes_combine = (R + T) * M * es + T * k * 8.0
    bytes_dbwd = (R + T) * M * es + T * shape.E * 4.0
    hbm = {}
    for name, nbytes, per_step in (("dispatch", bytes_dispatch, n_disp_per_step), ("combine", bytes_combine, 1),
                                   ("dispatch_bwd", bytes_dbwd, 1)):
        l, ms = prof[name]
        if l and ms > 0:
            gbs = nbytes * per_step * steps / (ms * 1e-3) / 1e9
            hbm[name] = {"launches": l, "avg_us": 1e3 * ms / l, "GB/s": gbs, "frac": gbs / PEAK_HBM_GBS}

    # the same kernels with the schedule serialised on one stream (no GEMM running beside them)
    hbm_alone = {}
    others_alone = {}
    cost_model = {}
    if not brief and not args.single_stream:
        keep = st.s1
        st.s1 = st.s0
        B.moe_profile_enable(True)
        for _ in range(3):
            st.step()
        torch.cuda.synchronize()
        B.moe_profile_enable(False)
        st.s1 = keep
        prof1 = B.moe_profile_read()
        for name, nbytes, per_step in (("dispatch", bytes_dispatch, n_disp_per_step), ("combine", bytes_combine, 1),
                                       ("dispatch_bwd", bytes_dbwd, 1)):
            l, ms = prof1[name]
            if l and ms > 0:
                gbs = nbytes * per_step * 3 / (ms * 1e-3) / 1e9
                hbm_alone[name] = {"avg_us": 1e3 * ms / l, "GB/s": gbs, "frac": gbs / PEAK_HBM_GBS}
        others_alone = {kd: prof1[kd][1] / 3 for kd in ("route", "slots", "gate_bwd")}

    mem = {}
    for mode in (0, 1, 2, 3, 4, 5):
        cfg = B.make_config(T, M, H, shape.E, k, shape.capacity_factor, n,
                            B.MOE_BF16 if shape.dtype == "bf16" else B.MOE_F32, mode)
        total, saved, temp, routing = B.moe_workspace_bytes(cfg)
        mem[f"mode{mode}"] = {"workspace": total, "saved_activations": saved, "temporaries": temp, "routing": routing}
        if mode >= 3:
            mem[f"mode{mode}"]["pinned_host"] = B.moe_offload_bytes(cfg)
    mem["max_memory_allocated_this_run"] = int(peak_alloc)
    mem["this_run_workspace"] = ws_bytes

    out = {
        "metric": "MoE layer fwd+bwd tokens/sec", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_events": ev_ms / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": f"{shape.name}: T={T} M={M} H={H} E={shape.E} k={k} cf={shape.capacity_factor}",
                   "n_partitions": n, "reuse_mode": reuse, "streams": 1 if args.single_stream else 2,
                   "hip_graph": bool(args.graph), "fuse_gather": int(fuse), "wgrad_group": int(group),
                   "weight_grads": "accumulated into zeroed buffers" if args.accumulate else "overwritten each step",
                   "kept_rows": R, "drop_rate": drop_rate},
        "tflops_model": flop_model / (ms_per_step * 1e-3) / 1e12,
        "tflops_executed": flop_exec / (ms_per_step * 1e-3) / 1e12,
        "roofline": roofline, "hbm_kernels_alone": hbm_alone, "hbm_kernels_in_pipeline": hbm,
        "hbm_kernels_note": "alone = schedule serialised on one stream: the kernel's own duration. In the two-stream "
                            "pipeline the GEMM workgroups are persistent and hold every CU for a whole GEMM, so a "
                            "permutation kernel queued beside a GEMM mostly waits for CUs and its event-to-event "
                            "time measures that wait, not its memory rate.",
        "memory_bytes": mem,
        "other_kernels_ms_per_step": {kd: prof[kd][1] / steps for kd in ("route", "slots", "gate_bwd")},
        "other_kernels_alone_ms_per_step": others_alone,
        "interference_and_cost_model": cost_model,
        "_kept_rows": R,
        "paper_context": "MPipeMoE reports up to 2.8x speedup and up to 47% less memory than FasterMoE on 64 A100 "
                         "GPUs (8 DGX A100); ratios on other hardware, not a target for this number",
    }
    if brief:
        out = {"workload": out["config"]["workload"], "n_partitions": n, "reuse_mode": reuse, "fuse_gather": int(fuse),
               "wgrad_group": int(group), "tokens_per_s": out["value"],
               "ms_per_step": out["ms_per_step"], "tflops_executed": out["tflops_executed"],
               "gemm_tflops": roofline["achieved"], "gemm_frac_of_peak": roofline["frac"],
               "drop_rate": drop_rate, "workspace_bytes": ws_bytes}
    del st
    torch.cuda.empty_cache()
    return out, shape, inp


def memory_report(args, shape, inp):
    """Peak device memory of one step per memory mode and partition count, measured (torch's allocator:
    the library itself allocates nothing, so this is inputs + outputs + the workspace the mode asks for)
    beside the analytic workspace and the paper's closed form for the saving (Section III-D, Eq. 5 with
    kept rows in place of tokens: activations of one pass shrink by R (2M (n-2)/n + H (n-1)/n) elements,
    and Eq. 4's temporaries by the same again)."""
    import torch
    from paper_2506_22175_amd import runner
    es = 2 if shape.dtype == "bf16" else 4
    rows = []
    ns = [n for n in (1, 2, 4, 8) if shape.T % n == 0]
    for n in ns:
        base_peak = None
        for mode, group in ((0, 0), (1, 0), (2, 0), (2, n)):
            if group and n < 4:
                continue
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            before = torch.cuda.memory_allocated()
            torch.cuda.reset_peak_memory_stats()
            st = runner.LayerState(shape.T, shape.M, shape.H, shape.E, shape.k, shape.capacity_factor, n, shape.dtype,
                                   mode, second_stream=not args.single_stream, grad_overwrite=1, wgrad_group=group)
            st.upload(inp)
            st.step()
            torch.cuda.synchronize()
            peak = torch.cuda.max_memory_allocated() - before
            R = n * st.C_p * shape.E                                  # rows of all partition buffers
            row = {"n_partitions": n, "reuse_mode": mode, "wgrad_group": group,
                   "workspace_bytes": int(st.ws_total), "saved_activation_bytes": int(st.ws_saved),
                   "temporary_bytes": int(st.ws_temp), "measured_peak_bytes": int(peak)}
            if mode == 0 and not group:
                base_peak, base_saved = peak, st.ws_saved
            elif base_peak is not None and not group:
                # Eq. 5: what sharing T_DI / T_DO (two buffers each) and, with recomputation, T_M (one buffer) saves
                eq5 = R * (2 * shape.M * max(n - 2, 0) / n + (shape.H * (n - 1) / n if mode == 2 else 0.0)) * es
                row["eq5_saving_bytes"] = int(eq5)
                row["measured_saving_bytes"] = int(base_peak - peak)
                row["saved_activation_saving_bytes"] = int(base_saved - st.ws_saved)
                row["achieved_over_theoretical"] = (base_peak - peak) / eq5 if eq5 > 0 else None
            elif base_peak is not None:
                row["measured_saving_bytes"] = int(base_peak - peak)
            rows.append(row)
            del st
    torch.cuda.empty_cache()
    return {"per_mode_and_partitioning": rows,
            "note": "measured_peak = torch.cuda.max_memory_allocated over one step, minus what was allocated before "
                    "(x, dy, y, dx, weights, float weight gradients, routing outputs and the workspace). "
                    "eq5_saving is the paper's forward-activation saving; the workspace also shares backward's "
                    "temporaries, which is why achieved_over_theoretical can exceed 1 (the paper reports about "
                    "95 % of its own model, Section V-C)"}


def granularity_report(args, shape, inp, reuse):
    """Algorithm 1 (adaptive pipeline granularity) on this workload's layer at several batch
    sizes: searches by timed trials where it must, answers from its range set where it can."""
    import torch
    from paper_2506_22175_amd import binding as B
    from paper_2506_22175_amd import runner
    cands = [1, 2, 4, 8]
    full = shape.T
    order = [full // 8, full // 4, full // 2, full, full * 3 // 8, full * 3 // 4]     # the last two fall between searched sizes
    g = B.GranHandle()
    rows = []
    for T in order:
        st = runner.LayerState(T, shape.M, shape.H, shape.E, shape.k, shape.capacity_factor, 1, shape.dtype, reuse,
                               second_stream=not args.single_stream, size_for_partitions=cands)
        st.upload({k_: (v[:T] if k_ in ("x", "dy") else v) for k_, v in inp.items()})
        known = B.moe_gran_lookup(g, T)
        row = {"T": T}
        if known == -1:
            best, ms = st.search_best_gran(cands, warmup=1, iters=3)
            B.moe_gran_record(g, T, best)
            row.update({"n": best, "how": "searched", "ms_per_step": dict(zip(map(str, cands), ms))})
        else:
            # answered from the range set; time the candidates anyway to check the answer
            best, ms = st.search_best_gran(cands, warmup=1, iters=3)
            row.update({"n": known, "how": "from range", "trial_best_n": best,
                        "ms_per_step": dict(zip(map(str, cands), ms))})
        rows.append(row)
        del st
        torch.cuda.empty_cache()
    out = {"candidates": cands, "queries": rows,
           "ranges": [{"lower": lo, "upper": up, "n": n} for lo, up, n in B.moe_gran_ranges(g)]}
    g.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--n", type=int, default=2, help="pipeline partitions")
    ap.add_argument("--reuse", type=int, default=2, help="0 keep all, 1 share buffers, 2 share + recompute")
    ap.add_argument("--wgrad-group", type=int, default=0,
                    help="partitions whose weight gradients are taken in one GEMM (0 or 1: every partition its own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single-stream", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=16384, help="tokens of the workload the CPU oracle is timed on")
    ap.add_argument("--graph", action="store_true", help="replay a captured HIP graph of the step (no per-kernel timing)")
    ap.add_argument("--accumulate", action="store_true",
                    help="weight gradients are added to the buffers (default: each step overwrites them)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="no HIP events around the kernels in the timed region (roofline fields are then empty)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--fuse-gather", action="store_true",
                    help="the first expert GEMM gathers its rows from the token-major input (no forward dispatch)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    out, shape, inp = measure(args, args.workload, args.n, args.reuse, args.steps, args.warmup,
                              fuse=1 if args.fuse_gather else 0, group=args.wgrad_group)
    kept_rows = out.pop("_kept_rows")
    if not args.no_sweep:
        # Section II-C's slowdown factors as real co-runs, and Eq. 10 with them (Section III-E)
        from paper_2506_22175_amd import measure as msr
        itf = msr.interference(shape, inp, args.n, args.reuse, wgrad_group=args.wgrad_group)
        units = args.n * (2 + 4 + (1 if args.reuse in (2, 5) else 0))
        co_r = min((r for r in itf["side_by_side"] if r["free_cus"] > 0), key=lambda r: r["step_ms"])["free_cus"]
        model = msr.strategy_model(shape, args.n, kept_rows, units, itf, co_r)
        model.pop("_speeds_struct")
        out["interference_and_cost_model"] = {
            "per_free_cus": itf, "model": model,
            "note": "alone = whole schedule on one stream, GEMMs on every compute unit; side_by_side = two streams "
                    "with free_cus units left to the permutations; sigma, mu = time alone / time side by side. "
                    "At free_cus = 0 mu is the time a permutation waits for a unit, not a co-run slowdown; the "
                    "model takes sigma and mu from the best free_cus > 0",
            "this_run": {"strategy": {0: "none", 2: "S4"}.get(args.reuse, "mode 1 (no row in Table II)"),
                         "measured_step_ms": out["ms_per_step"]}}
    if not args.no_sweep:
        # the other workloads of the set, a few steps each, for the record
        others = []
        for wl, n, mode, grp in (("small", 1, 2, 0), ("gpt", 1, 2, 0), ("gpt", 4, 2, 0), ("gpt", 4, 2, 2),
                                 ("skewed", 4, 2, 0), ("skewed", 4, 2, 2), ("large", 4, 2, 0), ("large", 4, 2, 2),
                                 ("large", 8, 2, 0), ("large", 8, 2, 4),
                                 (args.workload, args.n, 0, 0), (args.workload, args.n, 1, 0),
                                 (args.workload, args.n, 3, 0), (args.workload, args.n, 4, 0), (args.workload, args.n, 5, 0)):
            if wl == args.workload and n == args.n and mode == args.reuse and grp == args.wgrad_group:
                continue
            o, _, _ = measure(args, wl, n, mode, 5, 2, brief=True, group=grp)
            others.append(o)
        # mid-size workload: every partition count under the three on-device memory modes (speed and
        # workspace side by side: Section III-C's granularity against Section III-D's reuse)
        grid = []
        for n in (1, 2, 4, 8):
            for mode in (0, 1, 2):
                o, _, _ = measure(args, "gpt", n, mode, 5, 2, brief=True)
                grid.append({k_: o[k_] for k_ in ("n_partitions", "reuse_mode", "ms_per_step", "tokens_per_s",
                                                   "gemm_frac_of_peak", "workspace_bytes")})
        out["gpt_partitions_by_mode"] = grid
        # the same configuration with the other setting of the gathered first GEMM
        o, _, _ = measure(args, args.workload, args.n, args.reuse, 10, 3, brief=True, fuse=0 if args.fuse_gather else 1)
        out["gathered_first_gemm"] = {"this_run": int(args.fuse_gather), "other_setting": o}
        out["other_workloads"] = others
        # measured step of every strategy of Table II beside Eq. 10's prediction
        names = {0: "none", 2: "S4", 3: "S1", 4: "S2", 5: "S3"}
        eq10 = out.get("interference_and_cost_model", {}).get("model", {}).get("eq10", {})
        meas = {names[o["reuse_mode"]]: o["ms_per_step"] for o in others
                if o["workload"] == out["config"]["workload"] and o["n_partitions"] == args.n and o["reuse_mode"] in names
                and o["wgrad_group"] == 0}
        meas[names.get(args.reuse, "mode 1")] = out["ms_per_step"]
        if eq10:
            out["interference_and_cost_model"]["measured_vs_eq10_step_ms"] = {
                k_: {"measured": meas.get(k_), "eq10": v["step_ms"]} for k_, v in eq10.items()}
    if not args.no_sweep:
        out["memory_bytes"]["measured"] = memory_report(args, shape, inp)
        out["adaptive_granularity"] = granularity_report(args, shape, inp, args.reuse)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, inp, args.cpu_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
