"""Host-side checks that need no GPU: the library loads, exports every declared symbol,
rejects bad arguments before launching anything, and its host arithmetic (SOL bound,
tile schedule, selection table) is right."""
import ctypes
import itertools
import os
import re

import pytest

import oracle
import paper_2603_29010_amd as ucl
from paper_2603_29010_amd.binding import Epilogue, Tuning, UclError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ucl.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(ucl_[a-z0-9_]+)\s*\(", hdr))
    assert {"ucl_gemm", "ucl_batched_gemm", "ucl_grouped_gemm", "ucl_conv2d_fprop", "ucl_sol_bound"} <= names
    lib = ctypes.CDLL(ucl.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in ucl.h but not exported"


def test_sol_bound_reproduces_paper_worked_example():
    g = {}
    for line in open(os.path.join(GOLD, "sol_report_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [t.strip() for t in line.split("=")]
            g[k] = v
    n = int(g["n"])
    ratio = float(g["sm_clock_mhz"]) / float(g["max_sm_clock_mhz"])
    hw = dict(peak_flops_f32=float(g["tf32_peak_tflops_at_max"]) * 1e12, peak_flops_16bit=0.0,
              peak_bw=float(g["hbm_tbps"]) * 1e12, compute_clock_ratio=ratio)
    r = ucl.ucl_sol_bound("gemm", "f32", "f32", hw=hw, M=n, N=n, K=n)
    assert r["flops"] == int(g["total_flops"]) and r["bytes"] == int(g["total_bytes"])
    assert round(r["t_compute"] * 1e3, 3) == float(g["t_compute_ms"])
    assert round(r["t_mem"] * 1e3, 3) == float(g["t_mem_ms"])
    assert round(r["t_sol"] * 1e3, 3) == float(g["t_sol_ms"])
    assert abs(r["ridge"] - float(g["ridge"])) < 0.06 and r["compute_bound"] == 1
    assert abs(r["peak_flops"] / 1e12 - float(g["tf32_peak_tflops_effective"])) < 0.02
    # FP16 augmentation: FP16 tensor peak, traffic stays FP32
    hw["peak_flops_f32"] = float(g["fp16_peak_tflops_at_max"]) * 1e12
    r16 = ucl.ucl_sol_bound("gemm", "f32", "f32", hw=hw, M=n, N=n, K=n)
    assert round(r16["t_sol"] * 1e3, 4) == float(g["t_sol_ms_fp16"]) and r16["bytes"] == r["bytes"]


def test_sol_bound_matches_oracle_arithmetic_on_the_five_configs():
    cases = [
        (dict(op="gemm", dt_in="bf16", dt_out="bf16", M=256, N=256, K=256), 2 * 256 ** 3, 3 * 256 * 256 * 2 + 512, True),
        (dict(op="gemm", dt_in="bf16", dt_out="bf16", M=4096, N=4096, K=4096), 137438953472, 100671488, True),
        (dict(op="batched_gemm", dt_in="f16", dt_out="f32", batch=64, M=512, N=512, K=128), 4294967296, 83886080, False),
        (dict(op="conv2d_fprop", dt_in="bf16", dt_out="bf16", conv=(32, 56, 56, 64, 128, 3, 3, 1, 1, 1, 1, 1, 1)),
         14797504512, 64372992, None),
    ]
    for kw, flops, nbytes, has_bias in cases:
        steps = []
        if has_bias is True:
            steps = [("bias", 16, "bf16")]
        elif has_bias is None:
            steps = [("bias", 16, "bf16"), ("aux_load", 16, "bf16", 128), ("relu",)]
        r = ucl.ucl_sol_bound(epi=Epilogue(steps), **kw)
        assert r["flops"] == flops and r["bytes"] == nbytes, (kw, r)
        o = oracle.sol_bound(flops, nbytes, 2516.6e12, 1.0, 8.0e12)
        for k in ("t_compute", "t_mem", "t_sol", "ai", "ridge"):
            assert r[k] == pytest.approx(o[k], rel=1e-12)
        assert r["compute_bound"] == o["compute_bound"]
    # the two gradients: the same multiply-accumulates as fprop, read dy + (w | x), write (dx | dw)
    conv = (32, 56, 56, 64, 128, 3, 3, 1, 1, 1, 1, 1, 1)
    n_x, n_w, n_y = 32 * 56 * 56 * 64, 128 * 9 * 64, 32 * 56 * 56 * 128
    r = ucl.ucl_sol_bound("conv2d_dgrad", "bf16", "bf16", conv=conv)
    assert r["flops"] == 14797504512 and r["bytes"] == 2 * (n_y + n_w) + 2 * n_x
    r = ucl.ucl_sol_bound("conv2d_wgrad", "bf16", "f32", conv=conv)
    assert r["flops"] == 14797504512 and r["bytes"] == 2 * (n_y + n_x) + 4 * n_w
    t = ucl.ucl_select_tuning("conv2d_wgrad", "bf16", "f32", conv=conv)
    assert t["tile_m"] in (64, 128) and t["iterator"] == 0
    M_g = [128, 2048, 640]
    r = ucl.ucl_sol_bound("grouped_gemm", "bf16", "bf16", M_g=M_g, N=4096, K=1024)
    assert r["flops"] == sum(M_g) * 8388608 and r["bytes"] == sum(M_g) * 10240 + 3 * 4096 * 1024 * 2


def test_tile_map_is_a_bijection_and_matches_brute_enumeration():
    for tiles_m, tiles_n, raster in [([16], 16, 4), ([3, 0, 5, 1], 7, 2), ([1], 1, 1), ([5, 5, 5], 3, 8),
                                     ([9], 2, 16), ([2, 7], 5, 1)]:
        total = sum(tiles_m) * tiles_n
        seen = set()
        for wg in range(total):
            g, tm, tn = ucl.ucl_tile_map(tiles_m, tiles_n, raster, wg)
            assert 0 <= tm < tiles_m[g] and 0 <= tn < tiles_n
            seen.add((g, tm, tn))
        want = {(g, a, b) for g, m in enumerate(tiles_m) for a in range(m) for b in range(tiles_n)}
        assert seen == want
    # workgroups of one XCD (same id mod 8) get a contiguous run of the band order
    ids = [ucl.ucl_tile_map([16], 16, 4, wg) for wg in range(0, 256, 8)]
    assert {t[1] for t in ids} == {0, 1, 2, 3} and {t[2] for t in ids} == set(range(8))


def test_selection_table():
    t = ucl.ucl_select_tuning("gemm", "bf16", "bf16", M=4096, N=4096, K=4096)
    assert (t["tile_m"], t["tile_n"]) == (256, 256)
    t = ucl.ucl_select_tuning("gemm", "bf16", "bf16", M=256, N=256, K=256)
    assert (t["tile_m"], t["tile_n"]) == (64, 64)
    # memory-bound by the SOL model (short K, fp32 output): a tile of which two workgroups share a CU
    t = ucl.ucl_select_tuning("batched_gemm", "f16", "f32", batch=64, M=512, N=512, K=128)
    assert (t["tile_m"], t["tile_n"], t["tile_k"], t["stages"]) == (256, 128, 32, 3)
    # conv: 3x3 / stride 1 / pad 1 / 64 channels takes the resident-patch iterator (2), anything else the gather (1)
    t = ucl.ucl_select_tuning("conv2d_fprop", "bf16", "bf16", conv=(32, 56, 56, 64, 128, 3, 3, 1, 1, 1, 1, 1, 1))
    assert (t["tile_m"], t["tile_n"], t["tile_k"], t["stages"], t["iterator"]) == (256, 128, 32, 4, 2)
    t = ucl.ucl_select_tuning("conv2d_fprop", "bf16", "bf16", conv=(32, 56, 56, 64, 128, 3, 3, 1, 1, 2, 2, 1, 1))
    assert t["iterator"] == 1
    t = ucl.ucl_select_tuning("conv2d_fprop", "bf16", "bf16", conv=(32, 56, 56, 32, 128, 3, 3, 1, 1, 1, 1, 1, 1))
    assert t["iterator"] == 1
    assert ucl.ucl_select_tuning("gemm", "bf16", "bf16", M=512, N=512, K=512)["iterator"] == 0
    # operand layouts take part: a row-major B (contiguous along N, config 1) is served by the kernels
    # that copy its rows directly, and only those; the pick must be one of the variants built for it
    variants = [ucl.ucl_variant(i) for i in range(ucl.ucl_num_variants())]
    for (al, bl) in itertools.product(("k", "mn"), repeat=2):
        t = ucl.ucl_select_tuning("gemm", "bf16", "bf16", M=256, N=256, K=256, a_layout=al, b_layout=bl)
        served = [v for v in variants if v["op_class"] == 0 and v["dt_in"] == 2
                  and v["a_layout"] == (al == "mn") and v["b_layout"] == (bl == "mn")
                  and v["a_path"] != 1 and v["b_path"] != 1]
        assert served and any((v["tile_m"], v["tile_n"], v["tile_k"], v["stages"]) ==
                              (t["tile_m"], t["tile_n"], t["tile_k"], t["stages"]) for v in served), (al, bl, t)
    t = ucl.ucl_select_tuning("gemm", "bf16", "bf16", M=256, N=256, K=256, b_layout="mn")
    assert (t["tile_m"], t["tile_n"], t["tile_k"], t["stages"]) == (64, 64, 64, 4)
    with pytest.raises(UclError):
        ucl.ucl_select_tuning("grouped_gemm", "bf16", "bf16", M_g=[64], N=64, K=64, a_layout="mn")
    assert all(0 < v["lds_bytes"] <= 160 * 1024 for v in variants)
    assert all(v["op_class"] in (0, 1, 2, 3, 4) and v["dt_in"] in (1, 2, 3, 4) for v in variants)


def _err(fn, *a, **k):
    with pytest.raises(UclError) as e:
        fn(*a, **k)
    return e.value


def test_validation_rejects_before_any_launch():
    P = 4096  # a 16-byte aligned fake address: validation must fail before it is ever dereferenced
    ok = dict(A=P, dtA="bf16", a_rs=64, a_cs=1, B=P, dtB="bf16", b_rs=1, b_cs=64, D=P, dtD="bf16", d_rs=64, d_cs=1)

    def gemm(M=64, N=64, K=64, **over):
        a = dict(ok, **over)
        ucl.ucl_gemm(M, N, K, a["A"], a["dtA"], a["a_rs"], a["a_cs"], a["B"], a["dtB"], a["b_rs"], a["b_cs"],
                     a["D"], a["dtD"], a["d_rs"], a["d_cs"], a.get("epi"), a.get("tune"))

    assert _err(gemm, M=0).status == "UCL_ERR_INVALID_ARG"
    assert _err(gemm, A=0).status == "UCL_ERR_INVALID_ARG"
    e = _err(gemm, A=P + 2)
    assert e.status == "UCL_ERR_UNSUPPORTED" and "16-byte aligned" in e.message
    e = _err(gemm, K=60)
    assert e.status == "UCL_ERR_UNSUPPORTED" and "multiple of 8" in e.message
    assert _err(gemm, a_rs=60).status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, a_rs=32).status == "UCL_ERR_INVALID_ARG"          # rows would overlap
    assert _err(gemm, a_rs=3, a_cs=5).status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, dtA="f32").status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, dtB="f16").status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, d_cs=64, d_rs=1).status == "UCL_ERR_UNSUPPORTED"
    e = _err(gemm, tune=Tuning(512, 512, 64, 2))
    assert e.status == "UCL_ERR_WORKSPACE" and "LDS" in e.message
    assert _err(gemm, tune=Tuning(96, 96, 64, 2)).status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, tune=Tuning(128, 128, 48, 2)).status == "UCL_ERR_UNSUPPORTED"
    assert _err(gemm, epi=Epilogue([("bias", 0, "bf16")])).status == "UCL_ERR_INVALID_ARG"
    assert _err(gemm, epi=Epilogue([("clamp", 2.0, 1.0)])).status == "UCL_ERR_INVALID_ARG"
    assert _err(gemm, epi=Epilogue([(77,)])).status == "UCL_ERR_INVALID_ARG"
    assert _err(ucl.ucl_grouped_gemm, [64] * 300, 64, 64, P, "bf16", 64, 1, P, "bf16", 1, 64, P, "bf16", 64, 1).status == "UCL_ERR_INVALID_ARG"
    assert _err(ucl.ucl_grouped_gemm, [64, -1], 64, 64, P, "bf16", 64, 1, P, "bf16", 1, 64, P, "bf16", 64, 1).status == "UCL_ERR_INVALID_ARG"
    e = _err(ucl.ucl_conv2d_fprop, 1, 8, 8, 3, 8, 3, 3, 1, 1, 1, 1, 1, 1, P, "bf16", P, "bf16", P, "bf16")
    assert e.status == "UCL_ERR_UNSUPPORTED" and "multiple of 8" in e.message
    assert _err(ucl.ucl_conv2d_fprop, 1, 2, 2, 8, 8, 5, 5, 0, 0, 1, 1, 1, 1, P, "bf16", P, "bf16", P, "bf16").status == "UCL_ERR_INVALID_ARG"
    # the GEMM entry points ignore a valid iterator value and still reject an invalid one
    assert _err(gemm, M=0, tune=Tuning(0, 0, 0, 0, 0, 2)).status == "UCL_ERR_INVALID_ARG"     # (fails on M, not on the iterator)
    assert _err(gemm, tune=Tuning(0, 0, 0, 0, 0, 7)).status == "UCL_ERR_INVALID_ARG"
    # an explicit tuning that names only tile_k is still an explicit tuning
    e = _err(gemm, tune=Tuning(0, 0, 48, 0))
    assert e.status == "UCL_ERR_UNSUPPORTED" and "tile_k" in e.message
    # transform stage: out of place only -- any overlap of the two byte ranges is rejected
    T = ucl.ucl_transpose
    assert _err(T, 1, 64, 64, P, "f32", P, "f32").status == "UCL_ERR_INVALID_ARG"
    assert _err(T, 1, 64, 64, P, "f32", P + 64 * 64 * 4 - 4, "bf16").status == "UCL_ERR_INVALID_ARG"
    assert _err(T, 2, 64, 64, P + 64 * 64 * 2 * 2 - 2, "f32", P, "bf16").status == "UCL_ERR_INVALID_ARG"
    assert _err(T, 1, 64, 64, P, "f32", 0, "bf16").status == "UCL_ERR_INVALID_ARG"
    T(0, 64, 64, P, "f32", P, "f32")             # zero extents: nothing to do, nothing launched
    # grouped with every group empty is a no-op, not an error (nothing is launched)
    ucl.ucl_grouped_gemm([0, 0], 64, 64, P, "bf16", 64, 1, P, "bf16", 1, 64, P, "bf16", 64, 1)
