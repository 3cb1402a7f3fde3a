#!/usr/bin/env python3
"""Benchmark of libsparsecontract on one MI355X.

A "step" is one sc_execute of the whole hot path (output fill, CSF traversal, on-chip
temporary, consumer stage, cross-tile fix-up) of the FUSED schedule on one synthetic
workload, with every input already resident in HBM.  The default workload is the MTTKRP
configuration (50,000 x 20,000 x 10,000, 20 M Zipf(1.2) nonzeros, rank 32, fp32).

Prints ONE JSON line: effective GFLOP/s of the schedule (its own flop count, multiply and
add counted separately, over the measured step time), a `roofline` object for the
dominant kernel (algorithmic HBM bytes over its HIP-event-timed duration against 8 TB/s)
and a `cpu_baseline` object (the fp64 oracle timed on the host cores in the same run).
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

WORKLOAD_TEXT = {
    1: "configs[0]: TTM chain order 3, fp64, 200^3, 8,000 uniform nonzeros, L=M=8",
    2: "configs[1]: MTTKRP order 3, fp32, 50,000x20,000x10,000, 20M Zipf(1.2) nonzeros, rank 32",
    3: "configs[2]: TTM chain order 3, fp32, 100,000x50,000x20,000, 30M Zipf(1.1) nonzeros, L=M=16",
    4: "configs[3]: SDDMM->SpMM, fp32, 1Mx1M, 16M nonzeros (rows Zipf 1.3), K=L=64",
    5: "configs[4]: TTM chain order 4, fp32, 10,000^4, 50M Zipf(1.1) nonzeros, L=M=N=8",
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload id 1..5 (default 2, the headline)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fissioned", action="store_true")
    ap.add_argument("--no-linear", action="store_true", help="skip the LINEAR (unfactored) nest, the baseline the paper's speedups are quoted against")
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

    cfg = synth.config(args.config, args.scale)
    t0 = time.time()
    data = synth.generate(cfg, cache_dir=os.environ.get("TMPDIR", "/tmp") + "/sc_synth_cache")
    t_gen = time.time() - t0
    out_shape = synth.output_shape(cfg)

    def timed(con, steps, warmup):
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
        timed.stats = {"median": float(np.median(per_step)), "std": float(per_step.std()),
                       "min": float(per_step.min()), "max": float(per_step.max())}
        return marks[0].elapsed_time(marks[steps]) / steps

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

    t0 = time.time()
    fused = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                        sc.schedule("fused"), out_shape)
    t_plan = time.time() - t0
    flops, bytes_fused = sc.plan_model(fused.plan)
    ms = timed(fused, args.steps, args.warmup)
    ms_stats = dict(timed.stats)
    kt = kernel_times(fused, min(args.steps, 20))
    dom_name = max(kt, key=kt.get)
    dom_ms = kt[dom_name]
    # algorithmic bytes of the dominant kernel: the schedule's compulsory bytes minus the
    # output fill, which is a separate launch
    elem = 8 if cfg["dtype"] == "f64" else 4
    out_bytes = float(np.prod(out_shape)) * elem
    dom_bytes = bytes_fused  # the fused kernel reads every input once and writes the output once
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # HBM bytes per launch from stored FETCH_SIZE / WRITE_SIZE counter runs (calibrated against
    # a copy of known size); None when absent or taken from other kernel sources
    measured = traffic_store.lookup(f"{args.config}:{dom_name}") if args.scale == 1.0 else None

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
    else:
        stream_copy = None

    result = {
        "metric": "effective GFLOP/s of the fused schedule (schedule flops / step time), 1 MI355X",
        "value": flops / (ms * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "ms_per_step_stats": ms_stats,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg["dtype"],
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config] + (f" (scaled by {args.scale})" if args.scale != 1.0 else ""),
                   "schedule": "fused", "nnz": int(cfg["nnz"]), "tiles": sc.plan_tile_count(fused.plan)},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured["hbm_bytes"] if measured else None,
                     "algorithmic_bytes": dom_bytes, "kernel_ms": dom_ms},
        "kernels_ms": kt,
        "schedule_flops": flops,
        "algorithmic_gbs_whole_step": bytes_fused / (ms * 1e-3) / 1e9,
        "setup_s": {"generate": t_gen, "convert_plan_upload": t_plan},
    }
    if stream_copy:
        result["stream_copy"] = stream_copy
    del fused
    torch.cuda.empty_cache()

    if not args.no_fissioned:
        fis = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule("fissioned"), out_shape)
        _, bytes_fis = sc.plan_model(fis.plan)
        ms_f = timed(fis, max(5, args.steps // 2), 2)
        kt_f = kernel_times(fis, 5)
        result["fissioned"] = {"ms_per_step": ms_f, "kernels_ms": kt_f, "algorithmic_bytes": bytes_fis,
                               "workspace_bytes": fis.ws_bytes}
        trav = [n for n in kt_f if "traverse" in n or "sddmm" in n or "leaf" in n]
        if trav:
            n = trav[0]
            # traversal kernel of the fissioned schedule: streams the leaves once, writes T once
            off, rows, cols = sc.plan_intermediate(fis.plan, 0)
            tb = cfg["nnz"] * (4 + elem) + rows * 4 + rows * cols * elem
            result["fissioned"]["traversal"] = {"kernel": n, "algorithmic_bytes": tb, "ms": kt_f[n],
                                                "gbs": tb / (kt_f[n] * 1e-3) / 1e9,
                                                "frac": tb / (kt_f[n] * 1e-3) / 1e9 / HBM_PEAK_GBS}
        result["fused_vs_fissioned_speedup"] = ms_f / ms
        del fis
        torch.cuda.empty_cache()

    if not args.no_linear:
        # the unfactored nest on the same GPU: what the fused schedule is a rewrite of (few steps: it is slow by design)
        lin = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule("linear"), out_shape)
        flops_lin, _ = sc.plan_model(lin.plan)
        ms_l = timed(lin, max(3, min(args.steps, 10)), 1)
        result["linear"] = {"ms_per_step": ms_l, "nest_flops": flops_lin, "gflops": flops_lin / (ms_l * 1e-3) / 1e9}
        result["fused_vs_linear_speedup"] = ms_l / ms
        del lin
        torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        from oracle import oracle as o
        o.build()
        cores = o.max_threads()
        # bounded sample: a prefix of whole top-level slices holding about `budget` multiply-adds
        per_nnz = {"ttmc3": lambda r: r[0] * r[1], "mttkrp3": lambda r: r[0], "sddmm_spmm": lambda r: r[0] + r[1],
                   "ttmc4": lambda r: r[0] * r[1] * r[2]}[cfg["kind"]](cfg["ranks"])
        budget = 4e9
        take = int(min(cfg["nnz"], max(1, budget // per_nnz)))
        coords = data["coords"][:, :take]
        vals = data["vals"][:take]
        t0 = time.time()
        o.contract(cfg["kind"], coords, vals, cfg["dims"], data["factors"], nthreads=cores)
        t_cpu = time.time() - t0
        frac = take / cfg["nnz"]
        result["cpu_baseline"] = {
            "value": flops * frac / t_cpu / 1e9, "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"first {take} of {cfg['nnz']} nonzeros (leading slices), fp64 linear loop nest, one run, "
                      f"{t_cpu:.2f} s; value = schedule flops x sampled fraction / time",
            "seconds": t_cpu,
        }

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
