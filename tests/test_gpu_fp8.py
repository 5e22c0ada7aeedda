"""GPU parity of gemm / batched_gemm with fp8 inputs (e4m3, e5m2; fp32 accumulate) against the fp64
oracle: exact on small integers (exactly representable in both formats) over every fp8 variant,
ragged shapes and K tails; floating point with fused epilogues over the whole value range of the
formats; split-K; validation."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning
from paper_2603_29010_amd.workload import DeviceWorkload

import parity
from test_gpu_parity import T, built

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", ["e4m3", "e5m2"])
def test_fp8_gemm_exact_every_variant(dt):
    # ragged M and N; K = 208 = 3 * 64 + 16: the smallest K tail the 16-byte alignment allows
    for (M, N, K) in ((328, 264, 208), (72, 136, 16), (264, 72, 1040)):
        spec = synth.gemm_spec(M, N, K, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
        for tile in built(0, dt=dt):
            parity.check_exact(spec, T(*tile), label=f"fp8 {dt} {M}x{N}x{K} {tile}")
        parity.check_exact(spec, None, label=f"fp8 {dt} {M}x{N}x{K} table choice")


@pytest.mark.parametrize("dt", ["e4m3", "e5m2"])
@pytest.mark.parametrize("dt_out", ["bf16", "f32"])
def test_fp8_gemm_parity_with_epilogue(dt, dt_out):
    spec = synth.gemm_spec(520, 392, 528, dt_in=dt, dt_out=dt_out, epilogue=("bias", "gelu_tanh"))
    for tile in built(0, dt=dt):
        parity.check(spec, T(*tile), label=f"fp8 {dt} {tile}")
    # operands spread over the formats' whole exponent range (subnormals to the largest values)
    spec = synth.gemm_spec(136, 200, 256, dt_in=dt, dt_out="f32", dist="normal", scale=1.0, epilogue=(("scale", 0.5),))
    rng = np.random.default_rng(3)
    for key in ("A", "B"):
        codes = rng.integers(0, 256, spec[key].shape, dtype=np.uint8)
        vals = synth.bits_to_f64(codes, dt)
        codes[~np.isfinite(vals)] = 0x38                      # no NaN / inf inputs
        spec[key] = codes
    # (products of two large values exceed fp32's range only beyond 2^128: e5m2's 57344^2 * 256 does not)
    # signs are random and magnitudes span 2^-9 .. 448 (2^-16 .. 57344): the sums cancel heavily, so the
    # error is judged against the accumulation bound K 2^-24 sum|a||b| alone
    parity.check(spec, None, label=f"fp8 {dt} every code", mandated=False)


@pytest.mark.parametrize("dt", ["e4m3", "e5m2"])
def test_fp8_benchmark_size_every_row_tile(dt):
    # the 4096^3 row of the benchmark's widening table, in the launch configuration it times (the table's choice):
    # every output element must have been written, and two rows of every 128-row wave tile are compared with the oracle
    spec = synth.gemm_spec(4096, 4096, 4096, dt_in=dt, dt_out="bf16", scale=1.0 / 64, epilogue=("bias", "gelu_tanh"))
    rng = np.random.default_rng(11)
    rows = sorted(int(b * 128 + r) for b in range(32) for r in rng.choice(128, 2, replace=False))
    parity.check(spec, None, rows=rows, label=f"fp8 {dt} 4096^3")


@pytest.mark.parametrize("dt", ["e4m3", "e5m2"])
def test_fp8_grouped_exact_and_parity(dt):
    # per-group pointer tables with one-byte elements: empty groups, ragged groups, K tail (K = 208 = 3 * 64 + 16)
    M_g = [0, 264, 64, 1, 0, 712, 130]
    spec = synth.grouped_spec(M_g, 264, 208, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    tiles = built(1, dt=dt)
    assert len(tiles) >= 3
    for tile in tiles:
        parity.check_exact(spec, T(*tile), label=f"fp8 grouped {dt} {tile}")
    parity.check_exact(spec, None, label=f"fp8 grouped {dt} table choice")
    # floating point, per-group bias and residual through the pointer tables, bf16 output
    spec = synth.grouped_spec([300, 0, 520, 77], 392, 528, dt_in=dt, dt_out="bf16", epilogue=("bias", "aux_load", "silu"))
    for tile in tiles:
        parity.check(spec, T(*tile), label=f"fp8 grouped {dt} bias+residual+silu {tile}")


def test_fp8_grouped_rejects_row_major_b_and_odd_k():
    w = DeviceWorkload(synth.grouped_spec([64, 64], 64, 72, dt_in="e4m3", dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        w.run()                                               # K = 72 is not a multiple of 16
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    w = DeviceWorkload(synth.grouped_spec([64, 64], 64, 64, dt_in="e4m3", dt_out="f32", epilogue=(), integer=True, b_layout="row"))
    with pytest.raises(ucl.UclError) as e:
        w.run()
    assert e.value.status == "UCL_ERR_UNSUPPORTED" and "contiguous along K" in e.value.message


def test_fp8_batched_and_split_k():
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    spec = synth.batched_spec(3, 136, 72, 1040, dt_in="e4m3", dt_out="f32", epilogue=(), integer=True)
    for tile in built(0, dt="e4m3"):
        parity.check_exact(spec, T(*tile), label=f"fp8 batched {tile}")
        for mode in ("serial", "parallel"):
            tune = Tuning(*tile, split_k=mode, slices=3, workspace=ws.data_ptr(), workspace_bytes=ws.numel())
            parity.check_exact(spec, tune, label=f"fp8 batched split-K {mode} {tile}")


def test_fp8_validation_and_sol():
    P = 4096
    args = lambda **o: dict(dict(M=64, N=64, K=64, a=(64, 1), b=(1, 64), dtA="e4m3", dtB="e4m3"), **o)

    def call(M, N, K, a, b, dtA, dtB):
        ucl.ucl_gemm(M, N, K, P, dtA, a[0], a[1], P, dtB, b[0], b[1], P, "bf16", N, 1)
    for bad, word in ((args(K=72, a=(72, 1), b=(1, 72)), "multiples of 16"), (args(a=(1, 64)), "contiguous along K"),
                      (args(dtB="e5m2"), "same fp8 type"), (args(a=(72, 1)), "multiples of 16")):
        with pytest.raises(ucl.UclError) as e:
            call(**bad)
        assert e.value.status == "UCL_ERR_UNSUPPORTED" and word in e.value.message, (bad, e.value.message)
    with pytest.raises(ucl.UclError) as e:          # an fp8 OUTPUT is not built
        ucl.ucl_gemm(64, 64, 64, P, "e4m3", 64, 1, P, "e4m3", 1, 64, P, "e4m3", 64, 1)
    assert e.value.status == "UCL_ERR_INVALID_ARG"
    with pytest.raises(ucl.UclError) as e:
        ucl.ucl_conv2d_fprop(1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1, 1, 1, P, "e4m3", P, "e4m3", P, "bf16")
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    r = ucl.ucl_sol_bound("gemm", "e4m3", "bf16", M=4096, N=4096, K=4096)
    assert r["bytes"] == 2 * 4096 * 4096 + 2 * 4096 * 4096 and r["peak_flops"] == 5033.2e12
