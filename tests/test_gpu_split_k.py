"""GPU parity of split-K (`.with_split_k(mode, slices)`): slices of the K extent run as separate
workgroups, their fp32 partial tiles pass through a caller-provided workspace and are added in
slice order.  Exact on integer inputs over every variant and layout, odd K, both modes; floating
point against the oracle; serial and parallel bit-identical; workspace contract."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning, WORKSPACE_COUNTER_BYTES
from paper_2603_29010_amd.workload import DeviceWorkload

import parity
from oracle import run_spec as orc_run
from test_gpu_parity import built

pytestmark = pytest.mark.gpu

_WS = {}


def workspace(nbytes):
    """One zero-initialised device buffer, grown on demand (counters cleared through the library)."""
    ws = _WS.get("buf")
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(nbytes, 64 << 20), dtype=torch.uint8, device="cuda")
        ws.fill_(0xA5)                                   # garbage: only the library's own init may be relied on
        ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        _WS["buf"] = ws
    return ws


def split_tune(tile, mode, slices, nbytes=None):
    ws = workspace(64 << 20)
    return Tuning(*tile, split_k=mode, slices=slices, workspace=ws.data_ptr(),
                  workspace_bytes=ws.numel() if nbytes is None else nbytes)


def counters_are_zero():
    torch.cuda.synchronize()
    return int(workspace(0)[:WORKSPACE_COUNTER_BYTES].count_nonzero().item()) == 0


@pytest.mark.parametrize("mode", ["serial", "parallel"])
@pytest.mark.parametrize("slices", [2, 4, 8])
def test_split_k_exact_every_variant(mode, slices):
    # ragged M and N, K = 1000 = 15 * 64 + 40: the last slice is short and ends inside a k-tile
    spec = synth.gemm_spec(200, 136, 1000, dt_out="f32", epilogue=(), integer=True)
    for tile in built(0):
        parity.check_exact(spec, split_tune(tile, mode, slices), label=f"split-K {mode} x{slices} {tile}")
    assert counters_are_zero()


@pytest.mark.parametrize("a_layout,b_layout", [("row", "row"), ("col", "col"), ("col", "row")])
def test_split_k_exact_other_layouts(a_layout, b_layout):
    la, lb = (5 if a_layout == "col" else 0), (4 if b_layout == "row" else 0)
    spec = synth.gemm_spec(200, 136, 712, dt_out="f32", a_layout=a_layout, b_layout=b_layout, epilogue=(), integer=True)
    for tile in built(0, la=la, lb=lb):
        for mode in ("serial", "parallel"):
            parity.check_exact(spec, split_tune(tile, mode, 3), label=f"split-K {a_layout}/{b_layout} {mode} {tile}")
    # the register-transposing fallback kernels split as well
    for tile in built(0, la=int(a_layout == "col"), lb=int(b_layout == "row")):
        parity.check_exact(spec, split_tune(tile, "serial", 4), label=f"split-K fallback {a_layout}/{b_layout} {tile}")
    assert counters_are_zero()


def test_split_k_exact_batched_and_f16():
    spec = synth.batched_spec(3, 136, 72, 520, dt_out="f32", epilogue=(), integer=True)
    for tile in built(0, f16=1):
        for mode in ("serial", "parallel"):
            parity.check_exact(spec, split_tune(tile, mode, 5), label=f"split-K batched {mode} {tile}")
    assert counters_are_zero()


def test_split_k_parallel_plain_f32_padded_rows():
    # An empty chain with fp32 output and more than two slices: the sums are the result, written without a
    # finishing pass over the tiles.  N = 134 is no multiple of 4 and the rows of D are 136 apart: the last
    # vector of a row is cut short, and the padding, the rows past M and the space behind D stay untouched.
    M, N, K, ldd = 200, 134, 1000, 136
    spec = synth.gemm_spec(M, N, K, dt_out="f32", epilogue=(), integer=True)
    ref = orc_run.run(spec).reshape(M, N)
    w = DeviceWorkload(spec)
    for tile in built(0):
        for mode in ("parallel", "serial"):
            D = torch.full((M + 1, ldd), -777.0, dtype=torch.float32, device="cuda")
            ucl.ucl_gemm(M, N, K, w.A.data_ptr(), "bf16", *spec["a_strides"], w.B.data_ptr(), "bf16", *spec["b_strides"],
                         D.data_ptr(), "f32", ldd, 1, None, split_tune(tile, mode, 6), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            got = D.cpu().numpy().astype(np.float64)
            assert np.array_equal(got[:M, :N], ref), f"{mode} {tile}"
            assert (got[:M, N:] == -777.0).all() and (got[M] == -777.0).all(), f"{mode} {tile}: wrote outside D"
    assert counters_are_zero()


@pytest.mark.parametrize("dt_out,chain", [("bf16", ("bias", "silu")), ("f16", (("scale", 0.5), "bias", "gelu_erf")), ("f32", ("bias", "relu")),
                                          ("bf16", ("bias", "aux_load", "relu")), ("f32", ("aux_load",))])
def test_split_k_parallel_simple_chain_padded_rows(dt_out, chain):
    # Chains of the form act(alpha * acc + bias[n] + beta * R[m, n]) are finished by the reduction kernel itself (more than two slices):
    # the same bits as serial mode, where the tile kernel runs the chain; rows of D padded to 136 with N = 134, so the
    # last vector of a row is cut short and the padding must stay untouched.
    M, N, K, ldd = 200, 134, 1000, 136
    spec = synth.gemm_spec(M, N, K, dt_in="f16" if dt_out == "f16" else "bf16", dt_out=dt_out, epilogue=chain)
    ref, absacc = parity.oracle_result(spec)
    w = DeviceWorkload(spec)
    tdt = torch.float32 if dt_out == "f32" else torch.int16
    for tile in built(0, f16=int(dt_out == "f16")):
        bits = {}
        for mode in ("parallel", "serial"):
            D = torch.full((M + 1, ldd), 12345 if dt_out != "f32" else -777.0, dtype=tdt, device="cuda")
            ucl.ucl_gemm(M, N, K, w.A.data_ptr(), spec["dt_in"], *spec["a_strides"], w.B.data_ptr(), spec["dt_in"], *spec["b_strides"],
                         D.data_ptr(), dt_out, ldd, 1, w.epi, split_tune(tile, mode, 6), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            raw = D.cpu().numpy()
            assert (raw[:M, N:] == raw[M, 0]).all() and (raw[M] == raw[M, 0]).all(), f"{mode} {tile}: wrote outside D"
            bits[mode] = (raw if dt_out == "f32" else raw.view(np.uint16))[:M, :N].copy()
        assert np.array_equal(bits["parallel"], bits["serial"]), f"{tile}: parallel and serial differ"
        got = synth.bits_to_f64(np.ascontiguousarray(bits["parallel"]), dt_out)
        parity.compare(got.reshape(ref.shape), ref, absacc, spec, f"parallel x6 {tile}")
    assert counters_are_zero()


def test_split_k_more_slices_than_k_tiles_and_auto():
    # K = 72: two 64-wide ranges at most; a request for 8 slices is cut down to 2
    spec = synth.gemm_spec(72, 72, 72, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, split_tune((64, 64, 32, 3), "serial", 8), label="8 slices over K=72")
    # slices = 0: the library chooses (few tiles, long K)
    spec = synth.gemm_spec(136, 72, 4096, dt_out="f32", epilogue=(), integer=True)
    for mode in ("serial", "parallel"):
        parity.check_exact(spec, split_tune((0, 0, 0, 0), mode, 0), label=f"auto slices {mode}")
    nbytes, slices = ucl.ucl_workspace_size("gemm", "bf16", "f32", Tuning(split_k="serial"), M=136, N=72, K=4096)
    assert slices > 1 and nbytes > WORKSPACE_COUNTER_BYTES
    # slices = 1 and mode none are the plain kernel and need no workspace
    parity.check_exact(spec, Tuning(split_k="serial", slices=1), label="one slice")
    assert counters_are_zero()


@pytest.mark.parametrize("chain", [("bias", "gelu_tanh"), ("bias", "aux_load", "relu"), ("per_row_scale", "tanh")],
                         ids=lambda c: "-".join(c))
def test_split_k_parity_epilogue_runs_once_after_the_sum(chain):
    spec = synth.gemm_spec(264, 200, 2056, dt_out="bf16", epilogue=chain)
    ref, absacc = parity.oracle_result(spec)
    out = {}
    for mode in ("serial", "parallel"):
        for slices in (2, 7):
            w = DeviceWorkload(spec)
            w.run(tune=split_tune((128, 128, 64, 2), mode, slices))
            got = w.result()
            parity.compare(got, ref, absacc, spec, f"split-K {mode} x{slices}")
            out[(mode, slices)] = w.result_bits().copy()
    # the slices are added in slice order whoever does it: both modes agree bit for bit
    for slices in (2, 7):
        assert np.array_equal(out[("serial", slices)], out[("parallel", slices)])
    assert counters_are_zero()


def test_split_k_config1_class_deep_k():
    # few output tiles, deep K: the shape class split-K exists for; table choice + library's slice count
    spec = synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu"))
    parity.check(spec, split_tune((0, 0, 0, 0), "serial", 0), label="256x256x16384 serial auto")
    parity.check(spec, split_tune((0, 0, 0, 0), "parallel", 0), label="256x256x16384 parallel auto")


def test_split_k_repeated_calls_and_graph_replay():
    spec = synth.gemm_spec(200, 136, 1000, epilogue=("bias", "silu"))
    w = DeviceWorkload(spec)
    tune = split_tune((64, 64, 64, 4), "serial", 4)
    w.run(tune=tune)
    first = w.result_bits().copy()
    for _ in range(3):                                   # the counters were left at zero
        w.D.zero_()
        w.run(tune=tune)
        assert np.array_equal(w.result_bits(), first)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        w.run(tune=tune)
        w.run(tune=split_tune((64, 64, 64, 4), "parallel", 4))
    for rep in range(3):
        w.D.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(w.result_bits(), first), f"replay {rep}"
    assert counters_are_zero()


def test_split_k_serial_partials_are_never_stale():
    # Partial tiles pass between workgroups on different XCDs, each with its own L2.  The same workspace
    # region is written again and again with different data (three problems of one shape, alternating,
    # different slice counts): a reader that saw a line left in its L2 by an earlier call would give an
    # earlier call's sums.  Integer data: every call must reproduce its problem's result bit for bit.
    specs = [synth.gemm_spec(264, 200, 2048, dt_out="f32", epilogue=(), integer=True, seed=synth.BASE_SEED + 20 + i) for i in range(3)]
    works = [DeviceWorkload(sp) for sp in specs]
    refs = [parity.orc_run.run(sp) for sp in specs]
    assert not np.array_equal(refs[0], refs[1])
    for it in range(36):
        i = it % 3
        tile = ((64, 64, 64, 4), (128, 128, 64, 2), (256, 256, 64, 2))[(it // 3) % 3]
        works[i].D.fill_(float("nan"))
        works[i].run(tune=split_tune(tile, "serial", 2 + it % 7))
        got = works[i].result()
        assert np.array_equal(got, refs[i]), f"call {it}: problem {i}, tile {tile}: {np.count_nonzero(got != refs[i])} wrong elements"
    assert counters_are_zero()


def test_split_k_workspace_contract():
    spec = synth.gemm_spec(200, 136, 1000, dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    need, slices = ucl.ucl_workspace_size("gemm", "bf16", "f32", Tuning(64, 64, 32, 3, split_k="serial", slices=4), M=200, N=136, K=1000)
    assert slices == 4 and need == WORKSPACE_COUNTER_BYTES + 4 * (4 * 3) * 64 * 64 * 4
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=Tuning(64, 64, 32, 3, split_k="serial", slices=4))
    assert e.value.status == "UCL_ERR_WORKSPACE" and str(need) in e.value.message
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=split_tune((64, 64, 32, 3), "serial", 4, nbytes=need - 1))
    assert e.value.status == "UCL_ERR_WORKSPACE"
    w.run(tune=split_tune((64, 64, 32, 3), "serial", 4, nbytes=need))      # exactly enough
    ref = parity.orc_run.run(spec)
    assert np.array_equal(w.result(), ref)
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=Tuning(64, 64, 32, 3, split_k="none", slices=4))
    assert e.value.status == "UCL_ERR_INVALID_ARG"
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=Tuning(scheduler="stream_k"))                # the stream-K scheduler needs a workspace as well
    assert e.value.status == "UCL_ERR_WORKSPACE"
    g = DeviceWorkload(synth.grouped_spec([64, 64], 64, 256, dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        g.run(tune=split_tune((0, 0, 0, 0), "serial", 2))
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
