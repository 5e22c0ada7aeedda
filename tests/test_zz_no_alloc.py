"""The allocation-free split-K entry point (ucl_gemm_static_workspace: partial tiles and counters in
a workspace that is part of the library's device code) against ucl_gemm with a caller-provided
workspace: same kernels, same order of additions, so the outputs must agree bit for bit -- on two
calls in a row, the second on a smaller problem (the shared workspace keeps the first call's
contents), in both split-K modes; and both against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import STATIC_WORKSPACE_BYTES, Tuning
from paper_2603_29010_amd.workload import DeviceWorkload

import parity

pytestmark = pytest.mark.gpu


def run_static(w, tune):
    s = w.spec
    ucl.ucl_gemm_static_workspace(s["M"], s["N"], s["K"], w.A.data_ptr(), s["dt_in"], *s["a_strides"],
                                  w.B.data_ptr(), s["dt_in"], *s["b_strides"], w.D.data_ptr(), s["dt_out"],
                                  s["N"], 1, w.epi, tune, torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("mode", ["serial", "parallel"])
def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row(mode):
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    # first call: 4 x 3 tiles of 64x64, 6 slices; second call: smaller in every extent, fewer slices
    for (M, N, K, slices) in ((200, 136, 1544, 6), (72, 64, 520, 3)):
        spec = synth.gemm_spec(M, N, K, dt_out="bf16", epilogue=("bias", "gelu_tanh"))
        tile = (64, 64, 64, 4)
        a, b = DeviceWorkload(spec), DeviceWorkload(spec)
        a.run(tune=Tuning(*tile, split_k=mode, slices=slices, workspace=ws.data_ptr(), workspace_bytes=ws.numel()))
        run_static(b, Tuning(*tile, split_k=mode, slices=slices))
        want, got = a.result_bits(), b.result_bits()
        assert np.all(np.isfinite(b.result())), "unwritten output elements"
        assert np.array_equal(got, want), f"{mode} {M}x{N}x{K}: static workspace differs from the caller-provided one"
        ref, absacc = parity.oracle_result(spec)
        parity.compare(b.result(), ref, absacc, spec, f"static workspace {mode} {M}x{N}x{K}")


def test_static_workspace_exact_and_limits():
    spec = synth.gemm_spec(136, 200, 1000, dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    run_static(w, Tuning(split_k="serial", slices=4))
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
    # no split requested: this entry point is the split-K form
    with pytest.raises(ucl.UclError) as e:
        run_static(w, Tuning())
    assert e.value.status == "UCL_ERR_INVALID_ARG"
    # partial tiles beyond the static workspace: rejected before any launch, the output stays untouched
    big = synth.gemm_spec(1024, 1024, 512, dt_out="f32", epilogue=(), integer=True)
    need, slices = ucl.ucl_workspace_size("gemm", "bf16", "f32", Tuning(128, 128, 64, 2, split_k="serial", slices=8),
                                          M=1024, N=1024, K=512)
    assert need > STATIC_WORKSPACE_BYTES
    wb = DeviceWorkload(big)
    with pytest.raises(ucl.UclError) as e:
        run_static(wb, Tuning(128, 128, 64, 2, split_k="serial", slices=8))
    assert e.value.status == "UCL_ERR_WORKSPACE" and str(STATIC_WORKSPACE_BYTES) in e.value.message
    assert not np.any(np.isfinite(wb.result()))
