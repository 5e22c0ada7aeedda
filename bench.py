#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Headline workload (config 2 of the baseline): single GEMM M=N=K=4096, A row-major / B column-major
bf16, fp32 accumulate, fused bias + tanh-GELU epilogue, bf16 output.  A "step" is one pass of the
whole path: one ucl_gemm call (tile schedule, staged copies, MFMA mainloop, fused epilogue, store)
on inputs already resident in HBM.  Prints ONE JSON line on stdout.

  python bench.py [--steps K] [--warmup W] [--replays R] [--config {1..5}] [--headline-only]
                  [--no-cpu-baseline] [--eager]

Timing protocol (the same for every workload):
  1. spin-up: the workload is launched back to back for SPIN_UP_SECONDS regardless of --warmup, so
     that the engine clock has left its idle state and settled under load (the first ~100 launches
     after idle run 20-25 % slower); the engine clock is sampled from sysfs meanwhile;
  2. W untimed warm-up steps;
  3. K steps are recorded once into a HIP graph (kernel nodes only), replayed once untimed, then
     replayed R times, each replay bracketed by its own pair of HIP events on the launch stream;
     ms_per_step is the MEDIAN over the R replays of (replay time / K), with the minimum beside it.
     A further pass queues the R replays back to back inside one event pair ("sustained"): with a
     short graph (20 launches of 100 us) the host cannot submit graphs as fast as the GPU drains them
     and that figure shows the gaps (about 9 % there, 1 % with 100 launches per graph).
Memory-bound workloads rotate over enough distinct operand sets that no launch finds its inputs in
the 256 MB last-level cache.  The line carries a "configs" object with all five workloads, each with
its own roofline entry, unless --headline-only is given.
"""
import argparse
import glob
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2516.6      # dense bf16 / fp16, 256 CUs x 2.4 GHz x 4096 FLOP/clk
PEAK_HBM_GBPS = 8000.0
PEAK_SCLK_MHZ = 2400.0
SPIN_UP_SECONDS = 0.5
# HBM bytes moved per launch (read + written) as counted by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# each scaled by what the same counter reads for a plain 256 MiB device copy (2.000 and 1.000).
# Counters cannot be read from inside this process: these are the figures RECORDED in
# profiles/ucl_tile_kernel_*.txt (with the commands that produced them) for the kernels the selection
# table picks, not measurements of the run that prints them.
RECORDED_TRAFFIC_BYTES = {1: 1160248, 2: 235364923, 3: 84280114, 4: 525456226, 5: 66147739}
# The same for the rows of --widening (profiles/ucl_tile_kernel_widening_rows.txt; all launches of a step added up).
WIDENING_TRAFFIC_BYTES = {
    "gemm_4096x4096x4096_fp8_e4m3_rowcol_bias_gelu_tanh_bf16out": 134654126,
    "gemm_4096x4096x4096_fp8_e5m2_rowcol_bias_gelu_tanh_bf16out": 134633431,
    "grouped_gemm_16groups_n4096_k1024_fp8_e4m3_silu_bf16out": 321418944,
    "conv2d_dgrad_nhwc_32x56x56x64_from_128_3x3_bf16": 40370228,
    "conv2d_wgrad_nhwc_32x56x56x64_to_128_3x3_bf16_f32out_splitk_parallel": 106911202,
    "conv2d_wgrad_nhwc_32x56x56x64_to_128_3x3_bf16_f32out_splitk_serial": 66153438,
    "gemm_256x256x16384_bf16_bias_relu_no_split": 50682106,
    "gemm_256x256x16384_bf16_bias_relu_splitk_parallel": 25526644,
    "gemm_256x256x16384_bf16_bias_relu_splitk_serial": 25507331,
    "gemm_8192x8192x64_bf16_bias_relu_tile128_default_scheduler": 144121094,
    "gemm_256x256x16384_bf16_bias_relu_tile64_stream_k_scheduler": 25561483,
    "gemm_8192x8192x64_bf16_bias_relu_tile128_persistent_scheduler": 144121309,
}
WORKLOAD_NAMES = {
    1: "gemm_256x256x256_bf16_bias_relu",
    2: "gemm_4096x4096x4096_bf16_rowcol_bias_gelu_tanh",
    3: "batched_gemm_64x512x512x128_f16_scale_f32out",
    4: "grouped_gemm_16groups_N4096_K1024_bf16_silu",
    5: "conv2d_fprop_nhwc_32x56x56x64_to_128_3x3_bf16_bias_residual_relu",
}


class SclkSampler:
    """Polls the engine clock the driver reports (pp_dpm_sclk, the level marked '*') while a
    workload runs.  Best effort: where the file is missing or unreadable the result is None."""

    def __init__(self):
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.samples = []
        self._stop = threading.Event()
        self._thread = None

    def _read(self):
        for p in self.paths:
            try:
                for line in open(p):
                    if "*" in line:
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
            except (OSError, ValueError, IndexError):
                continue
        return None

    def __enter__(self):
        if self.paths:
            def loop():
                while not self._stop.is_set():
                    v = self._read()
                    if v:
                        self.samples.append(v)
                    time.sleep(0.02)
            self._thread = threading.Thread(target=loop, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        if self._thread:
            self._thread.join()

    def median(self):
        return statistics.median(self.samples) if self.samples else None


def timed_replays(run_step, steps, warmup, replays, use_graph=True):
    """Spin-up, warm-up, then `replays` timed passes of `steps` launches.  run_step(i) enqueues step
    i on torch's current stream.  Returns (per-step ms of every replay, launch kind, sclk MHz)."""
    import torch
    stream = torch.cuda.current_stream()
    with SclkSampler() as sclk:
        t0 = time.perf_counter()
        i = 0
        while SPIN_UP_SECONDS > 0 and time.perf_counter() - t0 < SPIN_UP_SECONDS:
            for _ in range(50):
                run_step(i)
                i += 1
            torch.cuda.synchronize()
    for i in range(warmup):
        run_step(i)
    torch.cuda.synchronize()
    launch, graph = "eager", None
    if use_graph:
        # the K launches recorded once into a HIP graph (kernel nodes only: the library issues no
        # memset or copy), so that the host's per-call cost cannot limit back-to-back short kernels
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(steps):
                    run_step(i)
            graph.replay()                       # untimed first replay
            torch.cuda.synchronize()
            launch = "hipgraph"
        except Exception as e:                   # capture unsupported: fall back to plain launches
            print(f"bench.py: graph capture failed ({e}); timing eager launches", file=sys.stderr)
            graph = None
    def one_replay():
        if graph is not None:
            graph.replay()
        else:
            for i in range(steps):
                run_step(i)
    # pass 1: the R replays queued back to back inside ONE event pair -- sustained throughput, nothing
    # but the work itself between the two events
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(replays):
        one_replay()
    b.record(stream)
    torch.cuda.synchronize()
    sustained = a.elapsed_time(b) / (steps * replays)
    # pass 2: every replay inside its own event pair (spread: median / min / max); a short graph pays
    # the gap between the event and the graph's first kernel once per replay
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
    for a, b in pairs:
        a.record(stream)
        one_replay()
        b.record(stream)
    torch.cuda.synchronize()
    return {"sustained": sustained, "per_replay": [a.elapsed_time(b) / steps for a, b in pairs]}, launch, sclk.median()


def launch_floor_us(steps, replays):
    """Per-launch time of the smallest launch the library can make (a one-element transform-stage
    call: one workgroup, one load, one store), timed like the workloads: the floor under any kernel."""
    import torch
    import paper_2603_29010_amd as ucl
    src = torch.zeros(4, dtype=torch.float32, device="cuda")
    dst = torch.zeros(4, dtype=torch.float32, device="cuda")

    def run(i):
        ucl.ucl_transpose(1, 1, 1, src.data_ptr(), "f32", dst.data_ptr(), "f32", torch.cuda.current_stream().cuda_stream)
    t, _, _ = timed_replays(run, steps, 5, replays)
    return statistics.median(t["per_replay"]) * 1e3


def time_workload(cfg, steps, warmup, replays, copies=None, use_graph=True):
    from paper_2603_29010_amd import synth
    from paper_2603_29010_amd.workload import DeviceWorkload
    spec = synth.config(cfg)
    probe = DeviceWorkload(spec, poison=False)
    sol = probe.sol()
    if copies is None:
        # memory-bound workloads: rotate over enough distinct operand sets that a launch cannot be
        # served from the 256 MB last-level cache left warm by the previous one
        # (at most 64 sets: the 0.4 MB problem of config 1 is bound by launch latency, not by where its operands sit)
        copies = 1 if sol["compute_bound"] else min(64, max(2, int(768e6 // sol["bytes"]) + 1))
    sets = [probe] + [DeviceWorkload(spec, poison=False) for _ in range(copies - 1)]
    timing, launch, sclk = timed_replays(lambda i: sets[i % copies].run(), steps, warmup, replays, use_graph)
    per_step = timing["per_replay"]
    ms = statistics.median(per_step)
    t = ms * 1e-3
    mfma = bool(sol["compute_bound"])
    tflops, gbps = sol["flops"] / t / 1e12, sol["bytes"] / t / 1e9
    res = {
        "workload": WORKLOAD_NAMES[cfg], "ms_per_step": ms, "ms_per_step_sustained": timing["sustained"],
        "ms_per_step_min": min(per_step), "ms_per_step_max": max(per_step), "tflops": tflops, "gbps": gbps, "flops": sol["flops"], "bytes": sol["bytes"],
        "t_sol_us": sol["t_sol"] * 1e6, "frac_of_sol": sol["t_sol"] / t,
        "buffer_sets": copies, "launch": launch, "kernel": probe.selected(),
        "roofline": {
            "bound": "mfma" if mfma else "hbm", "achieved": tflops if mfma else gbps,
            "peak": PEAK_MFMA_TFLOPS if mfma else PEAK_HBM_GBPS, "unit": "TFLOP/s" if mfma else "GB/s",
            "frac": (tflops / PEAK_MFMA_TFLOPS) if mfma else (gbps / PEAK_HBM_GBPS),
            "traffic": RECORDED_TRAFFIC_BYTES.get(cfg), "traffic_source": "recorded in profiles/ (rocprofv3 --pmc), not read in this run",
        },
        # integrity self-check (the paper's SOL-ceiling detector): nothing can beat the bound by > 10 %
        "below_sol_flag": bool(min(min(per_step), ms) * 1e-3 < 0.9 * sol["t_sol"]),
        "sclk_mhz_under_load": sclk,
    }
    if sclk:
        # the paper's report scales the compute peak by current / maximum clock
        scaled = probe.sol(hw={"peak_flops_16bit": PEAK_MFMA_TFLOPS * 1e12, "peak_flops_f32": 157.3e12,
                               "peak_bw": PEAK_HBM_GBPS * 1e9, "compute_clock_ratio": min(1.0, sclk / PEAK_SCLK_MHZ)})
        res["t_sol_clock_scaled_us"] = scaled["t_sol"] * 1e6
        res["frac_of_clock_scaled_sol"] = scaled["t_sol"] / t
    if spec["op"] == "grouped_gemm":
        res["sum_M"] = int(sum(spec["M_g"]))
    return res, spec, probe


def cpu_baseline(spec, cfg, probe):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload; what it computes is
    compared with the GPU output of the same rows (the test suite's two tolerances)."""
    from oracle import run_spec
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import parity
    probe.run()
    got_all = probe.result()
    if spec["op"] in ("gemm", "conv2d_fprop"):
        M = spec["M"]
        n = {1: M, 2: 4096, 5: 50176}.get(cfg, min(M, 1024))
        rows = list(range(0, M, max(1, M // n)))[:n]
        t0 = time.perf_counter()
        ref, absacc = run_spec.run(spec, rows=rows, want_abs=True)
        dt = time.perf_counter() - t0
        flops = 2.0 * len(rows) * spec["N"] * spec["K"]
        sample = f"{len(rows)} of {M} output rows (every {max(1, M // n)}th), all {spec['N']} columns"
        got = got_all[np.asarray(rows)]
        sub = spec
    else:
        import copy
        sub = copy.copy(spec)
        if spec["op"] == "batched_gemm":
            sub["batch"] = 16
            sub["A"], sub["B"] = spec["A"][:16], spec["B"][:16]
            flops = 2.0 * 16 * spec["M"] * spec["N"] * spec["K"]
            sample = f"16 of {spec['batch']} batches"
            got = got_all[:16]
        else:
            sub["M_g"] = [128] * len(spec["M_g"])
            offs = np.concatenate([[0], np.cumsum(spec["M_g"])])[:-1]
            sub["A"] = np.concatenate([spec["A"][o:o + 128] for o in offs])
            flops = 2.0 * 128 * len(spec["M_g"]) * spec["N"] * spec["K"]
            sample = "first 128 rows of each of the 16 groups"
            got = np.concatenate([got_all[o:o + 128] for o in offs])
        t0 = time.perf_counter()
        ref, absacc = run_spec.run(sub, want_abs=True)
        dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    out = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
           "sample": sample, "seconds": dt}
    try:
        out["gpu_vs_oracle_max_err"] = parity.compare(got.reshape(ref.shape), ref, absacc, sub, "bench")
        out["gpu_matches_oracle"] = bool(np.all(np.isfinite(got_all)))
    except AssertionError as e:
        out["gpu_matches_oracle"] = False
        out["gpu_vs_oracle_error"] = str(e)[:300]
    return out


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
    timing, launch, sclk = timed_replays(run, args.steps, args.warmup, args.replays, not args.eager)
    per_step = timing["per_replay"]
    ms = statistics.median(per_step)
    gbps = nbytes / (ms * 1e-3) / 1e9
    out = {
        "metric": "GB/s of algorithmic bytes (elements x (source + destination size)), transpose with conversion, 1 MI355X",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "replays": args.replays,
        "ms_per_step": ms, "ms_per_step_min": min(per_step),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w["name"], "buffer_sets": copies, "launch": launch, "bytes": nbytes,
                   "spin_up_seconds": SPIN_UP_SECONDS},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS,
                     "traffic": TRANSPOSE_TRAFFIC_BYTES, "traffic_source": "recorded in profiles/ (rocprofv3 --pmc), not read in this run"},
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


PEAK_FP8_TFLOPS = 5033.2


def bench_widening(args):
    """The rows beyond the five headline workloads (not part of the headline metric): fp8 GEMM and grouped GEMM, the two
    convolution gradients, a deep-K split-K GEMM and the persistent tile scheduler, each timed like the workloads above and set against
    its own roofline (ucl_sol_bound with the peak of its input type)."""
    import torch
    from paper_2603_29010_amd import synth
    from paper_2603_29010_amd.binding import Tuning
    from paper_2603_29010_amd.workload import DeviceWorkload
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    import paper_2603_29010_amd as ucl
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    split = lambda mode, slices=0: Tuning(split_k=mode, slices=slices, workspace=ws.data_ptr(), workspace_bytes=ws.numel())
    conv = dict(Nb=32, H=56, W=56, C=64, Ko=128, R=3, S=3, pad=(1, 1))
    cases = [
        ("gemm_4096x4096x4096_fp8_e4m3_rowcol_bias_gelu_tanh_bf16out",
         lambda: synth.gemm_spec(4096, 4096, 4096, dt_in="e4m3", dt_out="bf16", scale=1.0 / 64, epilogue=("bias", "gelu_tanh")), None),
        ("gemm_4096x4096x4096_fp8_e5m2_rowcol_bias_gelu_tanh_bf16out",
         lambda: synth.gemm_spec(4096, 4096, 4096, dt_in="e5m2", dt_out="bf16", scale=1.0 / 64, epilogue=("bias", "gelu_tanh")), None),
        ("grouped_gemm_16groups_n4096_k1024_fp8_e4m3_silu_bf16out",
         lambda: synth.grouped_spec(synth.grouped_sizes(16, synth.BASE_SEED + 4), 4096, 1024, dt_in="e4m3", scale=1.0 / 32,
                                    seed=synth.BASE_SEED + 4), None),
        ("conv2d_dgrad_nhwc_32x56x56x64_from_128_3x3_bf16", lambda: synth.conv_grad_spec("dgrad", **conv), None),
        ("conv2d_wgrad_nhwc_32x56x56x64_to_128_3x3_bf16_f32out_splitk_parallel",
         lambda: synth.conv_grad_spec("wgrad", dt_out="f32", **conv), split("parallel")),
        ("conv2d_wgrad_nhwc_32x56x56x64_to_128_3x3_bf16_f32out_splitk_serial",
         lambda: synth.conv_grad_spec("wgrad", dt_out="f32", **conv), split("serial")),
        ("gemm_256x256x16384_bf16_bias_relu_no_split",
         lambda: synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu")), None),
        ("gemm_256x256x16384_bf16_bias_relu_splitk_parallel",
         lambda: synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu")), split("parallel")),
        ("gemm_256x256x16384_bf16_bias_relu_splitk_serial",
         lambda: synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu")), split("serial")),
        # tile scheduler: the same 128x128x32x4 kernel, one workgroup per tile against one per CU slot
        ("gemm_8192x8192x64_bf16_bias_relu_tile128_default_scheduler",
         lambda: synth.gemm_spec(8192, 8192, 64, epilogue=("bias", "relu")), Tuning(128, 128, 32, 4)),
        ("gemm_256x256x16384_bf16_bias_relu_tile64_stream_k_scheduler",
         lambda: synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu")),
         Tuning(64, 64, 64, 4, scheduler="stream_k", workspace=ws.data_ptr(), workspace_bytes=ws.numel())),
        ("gemm_8192x8192x64_bf16_bias_relu_tile128_persistent_scheduler",
         lambda: synth.gemm_spec(8192, 8192, 64, epilogue=("bias", "relu")), Tuning(128, 128, 32, 4, scheduler="persistent")),
    ]
    out = {}
    for name, make, tune in cases:
        if args.only and args.only not in name:
            continue
        spec = make()
        w = DeviceWorkload(spec, poison=False)
        sol = w.sol()
        timing, launch, sclk = timed_replays(lambda i: w.run(tune=tune), args.steps, args.warmup, args.replays, not args.eager)
        ms = statistics.median(timing["per_replay"])
        t = ms * 1e-3
        mfma = bool(sol["compute_bound"])
        peak = (PEAK_FP8_TFLOPS if spec["dt_in"] in ("e4m3", "e5m2") else PEAK_MFMA_TFLOPS) if mfma else PEAK_HBM_GBPS
        ach = sol["flops"] / t / 1e12 if mfma else sol["bytes"] / t / 1e9
        out[name] = {"ms_per_step": ms, "ms_per_step_min": min(timing["per_replay"]), "tflops": sol["flops"] / t / 1e12,
                     "gbps": sol["bytes"] / t / 1e9, "t_sol_us": sol["t_sol"] * 1e6, "frac_of_sol": sol["t_sol"] / t,
                     "roofline": {"bound": "mfma" if mfma else "hbm", "achieved": ach, "peak": peak,
                                  "unit": "TFLOP/s" if mfma else "GB/s", "frac": ach / peak,
                                  "traffic": WIDENING_TRAFFIC_BYTES.get(name), "algorithmic_bytes": sol["bytes"],
                                  "traffic_source": "recorded in profiles/ (rocprofv3 --pmc), not read in this run"},
                     # (a split-K launch without a named tile picks its tile for the split launch: what the table would
                     # take for the unsplit problem is reported under a name of its own)
                     ("kernel_if_unsplit" if tune is not None and tune.c.split_k_mode else "kernel"):
                     w.selected() if tune is None or tune.c.split_k_mode else
                     dict(tune.as_dict(), scheduler=("default", "persistent", "stream_k")[tune.c.scheduler]),
                     "launch": launch, "sclk_mhz_under_load": sclk}
        if tune is not None and tune.c.split_k_mode:
            kw = w._problem_kwargs()
            out[name]["split_k"] = dict(zip(("workspace_bytes", "slices"),
                                            ucl.ucl_workspace_size(w.op, spec["dt_in"], spec["dt_out"], tune, **kw)))
        del w
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "widening rows: TFLOP/s or GB/s and fraction of the roofline per workload, 1 MI355X", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "replays": args.replays, "data": "synthetic", "workloads": out}))


def main():
    global SPIN_UP_SECONDS
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--replays", type=int, default=10, help="timed replays of the K-step graph (median reported)")
    ap.add_argument("--spin-up", type=float, default=SPIN_UP_SECONDS,
                    help="seconds of back-to-back launches before the warm-up (counter-collection runs pass 0)")
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--headline-only", action="store_true", help="skip the per-workload 'configs' object")
    ap.add_argument("--all", action="store_true", help="(default behaviour, kept for older command lines)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="plain launches instead of one captured HIP graph")
    ap.add_argument("--transpose", action="store_true",
                    help="time the pipeline transform stage (NCHW fp32 -> NHWC bf16) instead of a GEMM / conv workload")
    ap.add_argument("--widening", action="store_true",
                    help="time the rows beyond the headline workloads (fp8 GEMM, conv gradients, split-K) instead")
    ap.add_argument("--only", default="", help="with --widening: only the workloads whose name contains this text")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run 10 plain device copies of 256 MiB and exit (reference reading for the "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    SPIN_UP_SECONDS = args.spin_up
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (the hot path is one kernel on one GPU's share of the "
              "work); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.replays < 1 or args.steps < 1:
        print("bench.py: --steps and --replays must be positive", file=sys.stderr)
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
    if args.widening:
        bench_widening(args)
        return
    res, spec, probe = time_workload(args.config, args.steps, args.warmup, args.replays, use_graph=not args.eager)
    out = {
        "metric": "TFLOP/s and % of SOL (MFMA/HBM roofline) per GEMM/conv config, 1 MI355X",
        "value": res["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "replays": args.replays, "ms_per_step": res["ms_per_step"], "ms_per_step_sustained": res["ms_per_step_sustained"],
        "ms_per_step_min": res["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if spec["dt_in"] == "f16" else "bf16", "data": "synthetic",
        "config": {"workload": res["workload"], "frac_of_sol": res["frac_of_sol"], "t_sol_us": res["t_sol_us"],
                   "below_sol_flag": res["below_sol_flag"], "sclk_mhz_under_load": res["sclk_mhz_under_load"],
                   "t_sol_clock_scaled_us": res.get("t_sol_clock_scaled_us"),
                   "frac_of_clock_scaled_sol": res.get("frac_of_clock_scaled_sol"),
                   "buffer_sets": res["buffer_sets"], "launch": res["launch"], "kernel": res["kernel"],
                   "spin_up_seconds": SPIN_UP_SECONDS,
                   "timing": "ms_per_step / min: median / minimum over `replays` replays of a HIP graph of `steps` launches, one HIP event "
                             "pair per replay; sustained: the same replays queued back to back inside one event pair (includes the host's "
                             "gaps between graph launches, which show when the graph is short)"},
        "roofline": res["roofline"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, args.config, probe)
    if not args.headline_only:
        out["configs"] = {}
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                out["configs"][str(c)] = res
                continue
            del probe, spec
            torch.cuda.empty_cache()
            r, spec, probe = time_workload(c, args.steps, args.warmup, args.replays, use_graph=not args.eager)
            out["configs"][str(c)] = r
        # config 1 is bound by launch latency, not by either roofline: the floor it is measured against
        out["launch_floor_us"] = launch_floor_us(args.steps, args.replays)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
