#!/usr/bin/env python3
"""Benchmark of libsparsecontract on one MI355X.

A "step" is one sc_execute of the whole hot path (output fill, CSF traversal, on-chip
temporary, consumer stage, cross-tile fix-up) of the FUSED schedule on one synthetic
workload, with every input already resident in HBM.  The metric is per contraction, so the
default run measures all five benchmark workloads one after the other: the top-level
`value`, `roofline` and `cpu_baseline` are those of the largest one (the order-4 TTM chain,
50 M nonzeros), and `per_config` carries the same figures for each of the five.

Prints ONE JSON line.  Per workload: effective GFLOP/s of the schedule (its own flop count,
multiply and add counted separately, over the measured step time), a `roofline` object for
the dominant kernel (algorithmic HBM bytes over its HIP-event-timed duration against
8 TB/s), the FISSIONED schedule with its traversal kernel's achieved bandwidth, the LINEAR
(unfactored) nest, the two speedups, and the fp64 oracle timed on the host cores.
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

HBM_PEAK_GBS = 8000.0
HEADLINE = 5   # the largest single-GPU workload

WORKLOAD_TEXT = {
    1: "configs[0]: TTM chain order 3, fp64, 200^3, 8,000 uniform nonzeros, L=M=8",
    2: "configs[1]: MTTKRP order 3, fp32, 50,000x20,000x10,000, 20M Zipf(1.2) nonzeros, rank 32",
    3: "configs[2]: TTM chain order 3, fp32, 100,000x50,000x20,000, 30M Zipf(1.1) nonzeros, L=M=16",
    4: "configs[3]: SDDMM->SpMM, fp32, 1Mx1M, 16M nonzeros (rows Zipf 1.3), K=L=64",
    5: "configs[4]: TTM chain order 4, fp32, 10,000^4, 50M Zipf(1.1) nonzeros, L=M=N=8",
}

PAPER_CONTEXT = ("context only, other hardware and other baseline: the paper reports its fused schedules running "
                 "orders of magnitude faster than the default TACO schedules on 4x Intel Xeon E5-4650 "
                 "(32 cores, 2.7 GHz, 80 MB LLC, GCC 11.4 -O3 -ffast-math, median of 31 runs); it prints "
                 "no GFLOP/s or GB/s figure for these five workloads")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0,
                    help="measure only this workload (1..5); 6..10 = the headline workload plus one of the further workloads (all-mode TTMC and its rank sweep, kernel 8, kernel 2, uniform cases 1 and 2); default: everything, headline on the largest")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workloads (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fissioned", action="store_true")
    ap.add_argument("--no-linear", action="store_true",
                    help="skip the LINEAR (unfactored) nest, the baseline the paper's speedups are quoted against")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also queue and time the library's plain copy kernel (1 GiB), for counter runs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (sharding by top-level slice is "
              "described in DESIGN.md but not built)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd import synth
    from paper_2311_09549_amd import traffic as traffic_store
    from paper_2311_09549_amd.driver import Contraction

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    def timed(con, steps, warmup):
        """Mean and per-step statistics of `steps` executions after `warmup` untimed ones."""
        for _ in range(warmup):
            con.run()
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        marks[0].record()
        for i in range(steps):
            con.run()
            marks[i + 1].record()   # an event between steps costs nothing the stream waits for
        torch.cuda.synchronize()
        per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)])
        stats = {"median": float(np.median(per_step)), "std": float(per_step.std()),
                 "min": float(per_step.min()), "max": float(per_step.max())}
        return marks[0].elapsed_time(marks[steps]) / steps, stats

    def kernel_times(con, steps):
        """Average per-kernel milliseconds over `steps` profiled executions (HIP events
        recorded by the library on the launch stream around each kernel)."""
        sc.plan_set_profiling(con.plan, True)
        acc = {}
        order = []
        for _ in range(steps):
            con.run()
            torch.cuda.synchronize()
            for name, ms in sc.plan_kernel_times(con.plan):
                if name not in acc:
                    acc[name] = 0.0
                    order.append(name)
                acc[name] += ms
        sc.plan_set_profiling(con.plan, False)
        return {n: acc[n] / steps for n in order}

    def bench_config(cid):
        cfg = synth.config(cid, args.scale)
        t0 = time.time()
        data = synth.generate(cfg, cache_dir=os.environ.get("TMPDIR", "/tmp") + "/sc_synth_cache")
        t_gen = time.time() - t0
        out_shape = synth.output_shape(cfg)
        elem = 8 if cfg["dtype"] == "f64" else 4
        print(f"bench: config {cid} generated in {t_gen:.1f} s", file=sys.stderr, flush=True)

        t0 = time.time()
        fused = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                            sc.schedule("fused"), out_shape)
        t_plan = time.time() - t0
        flops, bytes_fused = sc.plan_model(fused.plan)
        ms, ms_stats = timed(fused, args.steps, args.warmup)
        kt = kernel_times(fused, min(args.steps, 10))
        dom_name = max(kt, key=kt.get)
        dom_ms = kt[dom_name]
        # algorithmic bytes of the dominant kernel: the fused kernel reads every input once and
        # writes the output once (the schedule's compulsory bytes)
        dom_bytes = bytes_fused
        achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
        # HBM bytes per launch from stored FETCH_SIZE / WRITE_SIZE counter runs (calibrated against a
        # copy of known size); None when absent or taken from other kernel sources
        measured = traffic_store.lookup(f"{cid}:{dom_name}") if args.scale == 1.0 else None
        rec = {
            "config_id": cid,
            "workload": WORKLOAD_TEXT[cid] + (f" (scaled by {args.scale})" if args.scale != 1.0 else ""),
            "dtype": cfg["dtype"],
            "nnz": int(cfg["nnz"]),
            "tiles": sc.plan_tile_count(fused.plan),
            "steps": args.steps,
            "ms_per_step": ms,
            "ms_per_step_stats": ms_stats,
            "schedule_flops": flops,
            "gflops": flops / (ms * 1e-3) / 1e9,
            "algorithmic_gbs_whole_step": bytes_fused / (ms * 1e-3) / 1e9,
            "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBS, "traffic": measured["hbm_bytes"] if measured else None,
                         "algorithmic_bytes": dom_bytes, "kernel_ms": dom_ms},
            "mfma_busy": measured.get("mfma_busy") if measured else None,
            "kernels_ms": kt,
            "setup_s": {"generate": t_gen, "convert_plan_upload": t_plan},
        }

        if not args.no_fissioned:
            fis = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                              sc.schedule("fissioned"), out_shape, share=fused)
            _, bytes_fis = sc.plan_model(fis.plan)
            ms_f, _ = timed(fis, max(5, args.steps // 2), 2)
            kt_f = kernel_times(fis, 5)
            rec["fissioned"] = {"ms_per_step": ms_f, "kernels_ms": kt_f, "algorithmic_bytes": bytes_fis,
                                "workspace_bytes": fis.ws_bytes}
            trav = [n for n in kt_f if "traverse" in n or "sddmm" in n or "leaf" in n]
            if trav:
                n = trav[0]
                # traversal kernel of the fissioned schedule: streams the leaves once, writes T once
                off, rows, cols = sc.plan_intermediate(fis.plan, 0)
                tb = cfg["nnz"] * (4 + elem) + rows * 4 + rows * cols * elem
                rec["fissioned"]["traversal"] = {"kernel": n, "algorithmic_bytes": tb, "ms": kt_f[n],
                                                 "gbs": tb / (kt_f[n] * 1e-3) / 1e9,
                                                 "frac": tb / (kt_f[n] * 1e-3) / 1e9 / HBM_PEAK_GBS}
            rec["fused_vs_fissioned_speedup"] = ms_f / ms
            del fis
            torch.cuda.empty_cache()

        if not args.no_linear:
            # the unfactored nest on the same GPU: what the fused schedule is a rewrite of (few steps: slow by design)
            lin = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                              sc.schedule("linear"), out_shape, share=fused)
            flops_lin, _ = sc.plan_model(lin.plan)
            ms_l, _ = timed(lin, max(3, min(args.steps, 5)), 1)
            rec["linear"] = {"ms_per_step": ms_l, "nest_flops": flops_lin, "gflops": flops_lin / (ms_l * 1e-3) / 1e9}
            rec["fused_vs_linear_speedup"] = ms_l / ms
            del lin
            torch.cuda.empty_cache()

        stream_copy = None
        if args.calibrate_copy:
            src = torch.empty(traffic_store.COPY_BYTES, dtype=torch.uint8, device="cuda:0").fill_(1)
            dst = torch.empty_like(src)
            stream = torch.cuda.current_stream().cuda_stream
            for _ in range(3):
                sc.stream_copy(dst, src, traffic_store.COPY_BYTES, stream)
            torch.cuda.synchronize()
            beg, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            beg.record()
            for _ in range(10):
                sc.stream_copy(dst, src, traffic_store.COPY_BYTES, stream)
            end.record()
            torch.cuda.synchronize()
            copy_ms = beg.elapsed_time(end) / 10
            # the library's plain copy kernel as a practical ceiling: bytes read + bytes written per second
            stream_copy = {"bytes_each_way": traffic_store.COPY_BYTES, "ms": copy_ms,
                           "gbs_read_plus_write": 2 * traffic_store.COPY_BYTES / (copy_ms * 1e-3) / 1e9}
            del src, dst
            rec["stream_copy"] = stream_copy

        del fused
        torch.cuda.empty_cache()

        if not args.no_cpu_baseline:
            from oracle import oracle as o
            o.build()
            cores = o.max_threads()
            # bounded sample: a prefix of whole top-level slices holding at most `budget` multiply-adds of the
            # linear nest per run (the whole workload when it is smaller), one warm-up run and three timed ones
            per_nnz = {"ttmc3": lambda r: r[0] * r[1], "mttkrp3": lambda r: r[0], "sddmm_spmm": lambda r: r[0] + r[1],
                       "ttmc4": lambda r: r[0] * r[1] * r[2]}[cfg["kind"]](cfg["ranks"])
            budget = 3e10
            take = int(min(cfg["nnz"], max(1, budget // per_nnz)))
            coords = data["coords"][:, :take]
            vals = data["vals"][:take]
            secs = o.time_contract(cfg["kind"], coords, vals, cfg["dims"], data["factors"], nthreads=cores, warmup=1, runs=3)
            t_cpu = float(np.median(secs))
            frac = take / cfg["nnz"]
            rec["cpu_baseline"] = {
                "value": flops * frac / t_cpu / 1e9, "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
                "sample": (f"first {take} of {cfg['nnz']} nonzeros (leading slices), fp64 linear loop nest, C call only, "
                           f"1 warm-up + median of 3 runs ({t_cpu:.3f} s); value = schedule flops x sampled fraction / time"),
                "seconds": t_cpu, "runs_s": secs,
            }
            rec["gpu_vs_cpu_oracle"] = rec["gflops"] / rec["cpu_baseline"]["value"]
        return rec

    K5_VARIANTS = [("schedule2_fused", "fused", []), ("schedule2_fissioned", "fissioned", ["T1(i,j,n)", "T2(i,m,n)"]),
                   ("schedule1", "fissioned", ["T(i,j,n)"]), ("schedule3", "fused", ["T(i,m,n)"]), ("linear", "linear", [])]
    CLASS_VARIANTS = [("fused", "fused", []), ("fissioned", "fissioned", []), ("linear", "linear", [])]

    def bench_next(cid, text, variants, steps, linear_flops=None, with_oracle=True, cfg=None):
        """A workload beyond the five benchmark ones: every listed schedule timed, the first one the reference of the
        speedups; kernels timed one by one; the oracle's perfectly nested loop timed when it runs in seconds."""
        cfg = cfg or synth.config(cid, args.scale)
        data = synth.generate(cfg, cache_dir=os.environ.get("TMPDIR", "/tmp") + "/sc_synth_cache")
        out_shape = synth.output_shape(cfg)
        rec = {"workload": text, "nnz": int(cfg["nnz"]), "ranks": list(cfg["ranks"]), "schedules": {}}
        first = None
        for name, kind, temps in variants:
            con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                              sc.schedule(kind, temps, [0] * len(temps)), out_shape, share=first)
            first = first or con
            flops, nbytes = sc.plan_model(con.plan)
            ms, stats = timed(con, steps, 2)
            kt = kernel_times(con, 5)
            dom = max(kt, key=kt.get)
            entry = {
                "ms_per_step": ms, "ms_per_step_stats": stats, "schedule_flops": flops, "gflops": flops / (ms * 1e-3) / 1e9,
                "kernels_ms": kt, "workspace_bytes": con.ws_bytes, "chosen": list(sc.plan_chosen(con.plan)),
                "roofline": {"bound": "hbm", "kernel": dom, "algorithmic_bytes": nbytes, "kernel_ms": kt[dom],
                             "achieved": nbytes / (kt[dom] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": nbytes / (kt[dom] * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None},
            }
            gemm = [n for n in kt if n.startswith("trailing_gemm")]
            if gemm:   # the GEMM-shaped stage on its own: its flops over its time against the fp32 matrix-core peak
                r_, m_ = cfg["ranks"][-2], cfg["ranks"][-1]
                gf = 2.0 * cfg["dims"][0] * r_ * m_
                entry["gemm_stage"] = {"kernel": gemm[0], "ms": kt[gemm[0]], "flops": gf, "tflops": gf / (kt[gemm[0]] * 1e-3) / 1e12,
                                       "frac_of_fp32_matrix_peak": gf / (kt[gemm[0]] * 1e-3) / 157.3e12}
            rec["schedules"][name] = entry
            if con is not first:
                del con
        del first
        torch.cuda.empty_cache()
        ref = variants[0][0]
        base = rec["schedules"][ref]["ms_per_step"]
        rec["speedup_of_" + ref + "_over"] = {k: v["ms_per_step"] / base for k, v in rec["schedules"].items()}
        if with_oracle and not args.no_cpu_baseline:
            from oracle import oracle as o
            o.build()
            cores = o.max_threads()
            secs = o.time_contract(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"], nthreads=cores, warmup=1, runs=3)
            t_cpu = float(np.median(secs))
            rec["cpu_baseline"] = {"seconds": t_cpu, "cores": cores, "kind": "oracle", "unit": "GFLOP/s",
                                   "value": (linear_flops or 0.0) / t_cpu / 1e9,
                                   "sample": "whole workload, the perfectly nested loop in fp64 (its own flop count), "
                                             "C call only, 1 warm-up + median of 3 runs"}
        return rec

    def bench_rank_sweep():
        """All-mode TTMC on the 4 M-nonzero tensor over dense sizes of the paper's auxiliary-memory table, schedule picked
        by the cost evaluator: time, the evaluator's choice, and the LDS footprint that decides how many workgroups share
        a compute unit (where the on-chip temporary stops fitting, the evaluator leaves the fused class)."""
        base = synth.config(6, args.scale)
        data0 = synth.generate(base, cache_dir=os.environ.get("TMPDIR", "/tmp") + "/sc_synth_cache")
        rows = []
        first = None
        for L, MN in [(16, 16), (64, 16), (128, 16), (16, 32), (64, 32), (128, 32), (16, 64), (64, 64), (128, 64), (16, 128), (128, 128)]:
            cfg = dict(base, ranks=(L, MN, MN))
            rng_cfg = synth.generate(dict(cfg, nnz=1, dims=base["dims"]))   # factors only (same seeds as a full draw)
            factors = rng_cfg["factors"]
            con = Contraction(cfg["expr"], data0["coords"], data0["vals"], cfg["dims"], factors, sc.schedule("auto"),
                              synth.output_shape(cfg))
            flops, nbytes = sc.plan_model(con.plan)
            mean_ms, st = timed(con, 7, 2)
            ms = st["median"]   # a point is a handful of launches: the median keeps one slow launch out of it
            text = sc.plan_describe(con.plan)
            chosen = [ln for ln in text.splitlines() if "<- chosen" in ln]
            rows.append({"L": L, "M": MN, "N": MN, "ms": ms, "mean_ms": mean_ms, "gflops": flops / (ms * 1e-3) / 1e9, "chosen": list(sc.plan_chosen(con.plan)),
                         "evaluator": chosen[0].strip() if chosen else None, "workspace_bytes": con.ws_bytes})
            del con
            torch.cuda.empty_cache()
        return rows

    cids = [5] if args.config >= 6 else [args.config] if args.config else [1, 2, 3, 4, 5]
    per_config = []
    for cid in cids:
        per_config.append(bench_config(cid))
        print(f"bench: config {cid} done: {per_config[-1]['ms_per_step']:.4f} ms/step, "
              f"{per_config[-1]['gflops']:.0f} GFLOP/s, roofline {per_config[-1]['roofline']['frac']:.3f}",
              file=sys.stderr, flush=True)
    head = next((r for r in per_config if r["config_id"] == HEADLINE), per_config[-1])

    result = {
        "metric": "effective GFLOP/s of the fused schedule (schedule flops / step time) per contraction, 1 MI355X",
        "value": head["gflops"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_stats": head["ms_per_step_stats"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "schedule": "fused", "nnz": head["nnz"], "tiles": head["tiles"]},
        "roofline": head["roofline"],
        "schedule_flops": head["schedule_flops"],
        "paper_context": PAPER_CONTEXT,
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    for k in ("fissioned", "fused_vs_fissioned_speedup", "linear", "fused_vs_linear_speedup", "kernels_ms", "mfma_busy",
              "stream_copy"):
        if k in head:
            result[k] = head[k]
    result["per_config"] = per_config
    if not args.config or args.config >= 6:
        nw = {}
        st = max(5, args.steps // 2)
        if args.config in (0, 6):
            L, M, N = synth.CONFIGS[6]["ranks"]
            nw["ttmc_all"] = bench_next(6, "all-mode TTMC A(l,m,n) (Table 2, kernel 5), fp32, 40,000x20,000x8,000, 4M Zipf(1.1) nonzeros, L=M=N=16",
                                        K5_VARIANTS, st, linear_flops=4.0 * L * M * N * synth.CONFIGS[6]["nnz"])
            nw["ttmc_all_rank_sweep"] = bench_rank_sweep()
        if args.config in (0, 7):
            R, M = synth.CONFIGS[7]["ranks"]
            nw["mttkrp_gemm"] = bench_next(7, "MTTKRP then GEMM A(i,m) (Table 2, kernel 8), fp32, the tensor of configs[1], R=32, M=64",
                                           CLASS_VARIANTS, st, linear_flops=4.0 * R * M * synth.CONFIGS[7]["nnz"])
        if args.config in (0, 8):
            nw["sddmm_spmm_gemm"] = bench_next(8, "SDDMM->SpMM then GEMM A(i,m) (Table 2, kernel 2), fp32, the matrix of configs[3], K=L=M=64",
                                               CLASS_VARIANTS[:2], st, with_oracle=False)
        if args.config in (0, 9):
            nw["ttmc_all_uniform_case1"] = bench_next(9, "all-mode TTMC, motivating case 1 of Section 3: uniform 1800x800x1000, sparsity 0.008, L,M,N=64,16,32 "
                                                         "(the paper's Figure 2 schedules on 32 Xeon cores: 2.48 s / 6.26 s / 32.40 s)", K5_VARIANTS, 5,
                                                      with_oracle=False)
        if args.config in (0, 10):
            nw["ttmc_all_uniform_case2"] = bench_next(10, "all-mode TTMC, motivating case 2 of Section 3: uniform 1800x1600x2000, sparsity 0.002, L,M,N=64,16,32 "
                                                          "(the paper's Figure 2 schedules on 32 Xeon cores: 10.20 s / 8.60 s / 33.51 s)", K5_VARIANTS, 5,
                                                       with_oracle=False)
        result["next_workloads"] = nw
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
