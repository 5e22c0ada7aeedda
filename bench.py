#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Default workload (config 2 of the baseline): single GEMM M=N=K=4096, A row-major / B column-major
bf16, fp32 accumulate, fused bias + tanh-GELU epilogue, bf16 output.  A "step" is one pass of the
whole path: one ucl_gemm call (tile schedule, staged copies, MFMA mainloop, fused epilogue, store)
on inputs already resident in HBM.  Prints ONE JSON line on stdout.

  python bench.py [--steps K] [--warmup W] [--config {1..5}] [--all] [--no-cpu-baseline]

--all adds a "configs" object with the other four workloads (each timed the same way, HBM-cold by
rotating over distinct buffer sets for the memory-bound ones).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2516.6      # dense bf16 / fp16, 256 CUs x 2.4 GHz x 4096 FLOP/clk
PEAK_HBM_GBPS = 8000.0
# HBM bytes moved per launch (read + written) as counted by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# each scaled by what the same counter reads for a plain 256 MiB device copy (2.000 and 1.000); the
# runs and their commands are recorded in profiles/ucl_tile_kernel_*.txt.  Counters cannot be read
# from inside this process, so these are the recorded figures for the kernels the selection table
# picks for each workload.
MEASURED_TRAFFIC_BYTES = {1: 1117221, 2: 235344518, 3: 84282176, 4: 525390133, 5: 66129995}
WORKLOAD_NAMES = {
    1: "gemm_256x256x256_bf16_bias_relu",
    2: "gemm_4096x4096x4096_bf16_rowcol_bias_gelu_tanh",
    3: "batched_gemm_64x512x512x128_f16_scale_f32out",
    4: "grouped_gemm_16groups_N4096_K1024_bf16_silu",
    5: "conv2d_fprop_nhwc_32x56x56x64_to_128_3x3_bf16_bias_residual_relu",
}


def time_workload(cfg, steps, warmup, copies=None, use_graph=True):
    """Time `steps` back-to-back launches with HIP events on the launch stream."""
    import torch
    from paper_2603_29010_amd import synth
    from paper_2603_29010_amd.workload import DeviceWorkload
    spec = synth.config(cfg)
    probe = DeviceWorkload(spec, poison=False)
    sol = probe.sol()
    if copies is None:
        # memory-bound workloads: rotate over enough distinct operand sets that a launch cannot be
        # served from the 256 MB last-level cache left warm by the previous one
        copies = 1 if sol["compute_bound"] else max(2, int(768e6 // sol["bytes"]) + 1)
    sets = [probe] + [DeviceWorkload(spec, poison=False) for _ in range(copies - 1)]
    for i in range(warmup):
        sets[i % copies].run()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    launch = "eager"
    graph = None
    if use_graph:
        # record the K launches once into a HIP graph (kernel nodes only: the library issues no memset
        # or copy), so that the host's per-call cost cannot limit back-to-back short kernels
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(steps):
                    sets[i % copies].run()
            graph.replay()                       # untimed first replay
            torch.cuda.synchronize()
            launch = "hipgraph"
        except Exception as e:                   # capture unsupported: fall back to plain launches
            print(f"bench.py: graph capture failed ({e}); timing eager launches", file=sys.stderr)
            graph = None
    stream = torch.cuda.current_stream()
    start.record(stream)
    if graph is not None:
        graph.replay()
    else:
        for i in range(steps):
            sets[i % copies].run()
    stop.record(stream)
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / steps
    t = ms * 1e-3
    res = {
        "workload": WORKLOAD_NAMES[cfg], "ms_per_step": ms, "tflops": sol["flops"] / t / 1e12,
        "gbps": sol["bytes"] / t / 1e9, "flops": sol["flops"], "bytes": sol["bytes"],
        "t_sol_us": sol["t_sol"] * 1e6, "frac_of_sol": sol["t_sol"] / t,
        "bound": "mfma" if sol["compute_bound"] else "hbm", "buffer_sets": copies, "launch": launch,
    }
    if spec["op"] == "grouped_gemm":
        res["sum_M"] = int(sum(spec["M_g"]))
    # integrity self-check (the paper's SOL-ceiling detector): nothing can beat the bound by > 10 %
    res["below_sol_flag"] = bool(t < 0.9 * sol["t_sol"])
    return res, spec, probe


def cpu_baseline(spec, cfg):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import run_spec
    import numpy as np
    if spec["op"] in ("gemm", "conv2d_fprop"):
        M = spec["M"]
        n = {1: M, 2: 4096, 5: 50176}.get(cfg, min(M, 1024))
        rows = list(range(0, M, max(1, M // n)))[:n]
        t0 = time.perf_counter()
        run_spec.run(spec, rows=rows)
        dt = time.perf_counter() - t0
        flops = 2.0 * len(rows) * spec["N"] * spec["K"]
        sample = f"{len(rows)} of {M} output rows (every {max(1, M // n)}th), all {spec['N']} columns"
    else:
        import copy
        sub = copy.copy(spec)
        if spec["op"] == "batched_gemm":
            sub["batch"] = 16
            sub["A"], sub["B"] = spec["A"][:16], spec["B"][:16]
            flops = 2.0 * 16 * spec["M"] * spec["N"] * spec["K"]
            sample = f"16 of {spec['batch']} batches"
        else:
            sub["M_g"] = [128] * len(spec["M_g"])
            offs = np.concatenate([[0], np.cumsum(spec["M_g"])])[:-1]
            sub["A"] = np.concatenate([spec["A"][o:o + 128] for o in offs])
            flops = 2.0 * 128 * len(spec["M_g"]) * spec["N"] * spec["K"]
            sample = "first 128 rows of each of the 16 groups"
        t0 = time.perf_counter()
        run_spec.run(sub)
        dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": sample, "seconds": dt}


TRANSPOSE_WORKLOAD = {"name": "transpose_nchw_to_nhwc_64x256x56x56_f32_to_bf16", "batch": 64, "rows": 256, "cols": 56 * 56,
                      "dt_src": "f32", "dt_dst": "bf16"}
TRANSPOSE_TRAFFIC_BYTES = 308402805


def bench_transpose(args):
    """The pipeline transform stage (a widening row, not one of the five headline workloads):
    NCHW fp32 -> NHWC bf16 of a [64, 256, 56, 56] activation tensor, HBM-cold rotation."""
    import numpy as np
    import torch
    import paper_2603_29010_amd as ucl
    from paper_2603_29010_amd import synth
    w = TRANSPOSE_WORKLOAD
    n = w["batch"] * w["rows"] * w["cols"]
    nbytes = n * (synth.itemsize(w["dt_src"]) + synth.itemsize(w["dt_dst"]))
    copies = max(2, int(768e6 // nbytes) + 1)
    host = synth.normal(synth.BASE_SEED + 6, 1, n).astype(np.float32)
    srcs = [torch.from_numpy(host).cuda() for _ in range(copies)]
    dsts = [torch.empty(n, dtype=torch.int16, device="cuda") for _ in range(copies)]

    def run(i):
        ucl.ucl_transpose(w["batch"], w["rows"], w["cols"], srcs[i % copies].data_ptr(), w["dt_src"],
                          dsts[i % copies].data_ptr(), w["dt_dst"], torch.cuda.current_stream().cuda_stream)
    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    launch = "eager"
    graph = None
    if not args.eager:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(args.steps):
                run(i)
        graph.replay()
        torch.cuda.synchronize()
        launch = "hipgraph"
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    stream = torch.cuda.current_stream()
    start.record(stream)
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            run(i)
    stop.record(stream)
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / args.steps
    gbps = nbytes / (ms * 1e-3) / 1e9
    out = {
        "metric": "GB/s of algorithmic bytes (elements x (source + destination size)), transpose with conversion, 1 MI355X",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w["name"], "buffer_sets": copies, "launch": launch, "bytes": nbytes},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS,
                     "traffic": TRANSPOSE_TRAFFIC_BYTES},
    }
    if not args.no_cpu_baseline:
        import oracle
        sample_b = w["batch"]
        x = host[:sample_b * w["rows"] * w["cols"]].reshape(sample_b, w["rows"], w["cols"])
        t0 = time.perf_counter()
        oracle.round_to(oracle.transpose(x, "f32", sample_b, w["rows"], w["cols"]), "bf16")
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nbytes * sample_b / w["batch"] / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"{sample_b} of {w['batch']} batches", "seconds": dt}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--all", action="store_true", help="also time the other four workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="plain launches instead of one captured HIP graph")
    ap.add_argument("--transpose", action="store_true",
                    help="time the pipeline transform stage (NCHW fp32 -> NHWC bf16) instead of a GEMM / conv workload")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run 10 plain device copies of 256 MiB and exit (reference reading for the "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (the hot path is one kernel on one GPU's share of the "
              "work); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 256 << 20, "copy_bytes_written": 256 << 20, "copies": 10}))
        return
    import paper_2603_29010_amd as ucl
    if not os.path.exists(ucl.library_path()):
        print("bench.py: libucl.so is not built (python -m paper_2603_29010_amd.build)", file=sys.stderr)
        sys.exit(1)

    if args.transpose:
        bench_transpose(args)
        return
    res, spec, _ = time_workload(args.config, args.steps, args.warmup, use_graph=not args.eager)
    mfma = res["bound"] == "mfma"
    roofline = {
        "bound": res["bound"],
        "achieved": res["tflops"] if mfma else res["gbps"],
        "peak": PEAK_MFMA_TFLOPS if mfma else PEAK_HBM_GBPS,
        "unit": "TFLOP/s" if mfma else "GB/s",
        "frac": (res["tflops"] / PEAK_MFMA_TFLOPS) if mfma else (res["gbps"] / PEAK_HBM_GBPS),
        "traffic": MEASURED_TRAFFIC_BYTES.get(args.config),
    }
    out = {
        "metric": "TFLOP/s and % of SOL (MFMA/HBM roofline) per GEMM/conv config, 1 MI355X",
        "value": res["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if spec["dt_in"] == "f16" else "bf16", "data": "synthetic",
        "config": {"workload": res["workload"], "frac_of_sol": res["frac_of_sol"], "t_sol_us": res["t_sol_us"],
                   "buffer_sets": res["buffer_sets"], "launch": res["launch"]},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, args.config)
    if args.all:
        out["configs"] = {}
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                out["configs"][str(c)] = res
                continue
            r, _, _ = time_workload(c, args.steps, args.warmup, use_graph=not args.eager)
            out["configs"][str(c)] = r
    print(json.dumps(out))


if __name__ == "__main__":
    main()
