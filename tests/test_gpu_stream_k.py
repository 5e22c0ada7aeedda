"""GPU parity of the stream-K tile scheduler (`.with_scheduler(tile=stream_k)`): every workgroup of a resident
grid takes an equal run of (tile, 64-wide k range) iterations; parts of tiles pass through the caller's workspace
and the workgroup that delivers a tile's last part adds them up in k order and runs the epilogue.  Exact on
integer inputs for every variant built with it -- tiles cut into many parts, whole tiles between two parts, one
k step per tile, K tails, batches -- floating point with fused epilogues against the oracle, bit-identical from
run to run with the workspace reused, workspace contract, rejections."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning, WORKSPACE_COUNTER_BYTES
from paper_2603_29010_amd.workload import DeviceWorkload

import parity
from test_gpu_parity import built

pytestmark = pytest.mark.gpu

_WS = {}


def workspace():
    ws = _WS.get("buf")
    if ws is None:
        ws = torch.empty(192 << 20, dtype=torch.uint8, device="cuda")
        ws.fill_(0xA5)                                   # garbage: only the library's own init may be relied on
        ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        _WS["buf"] = ws
    return ws


def SK(*tile, nbytes=None):
    ws = workspace()
    return Tuning(*tile, scheduler="stream_k", workspace=ws.data_ptr(), workspace_bytes=ws.numel() if nbytes is None else nbytes)


def counters_are_zero():
    torch.cuda.synchronize()
    return int(workspace()[:WORKSPACE_COUNTER_BYTES].count_nonzero().item()) == 0


TILES = [(t, "bf16") for t in built(0, scheduler=2)] + [(t, "f16") for t in built(0, f16=1, scheduler=2)]


def test_stream_k_variants_are_listed():
    assert built(0, scheduler=2) and built(0, f16=1, scheduler=2)


@pytest.mark.parametrize("tile,dt", TILES)
def test_stream_k_exact_few_tiles_deep_k(tile, dt):
    # 4 (128x128) or 12 (64x64) tiles of 32 k steps each over a few hundred workgroups: every tile is cut into many
    # parts, every workgroup holds a single part; ragged M and N, K = 1992 = 31 * 64 + 8 (a tail in the last part)
    spec = synth.gemm_spec(200, 136, 1992, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, SK(*tile), label=f"stream-K deep K {tile}")
    assert counters_are_zero()


@pytest.mark.parametrize("tile,dt", TILES)
def test_stream_k_exact_many_tiles(tile, dt):
    # more tiles than workgroups: a workgroup's run is the end of a tile, whole tiles, the start of a tile
    # (K = 200: four k steps per tile, the last one short)
    spec = synth.gemm_spec(3700, 3600, 200, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, SK(*tile), label=f"stream-K many tiles {tile}")
    assert counters_are_zero()


@pytest.mark.parametrize("tile,dt", TILES)
def test_stream_k_exact_one_step_per_tile_and_batches(tile, dt):
    # K = 40: one k step per tile, nothing is ever cut; then batches whose tiles follow one another in the run
    spec = synth.gemm_spec(1000, 900, 40, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, SK(*tile), label=f"stream-K K=40 {tile}")
    spec = synth.batched_spec(7, 328, 200, 712, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, SK(*tile), label=f"stream-K batched {tile}")
    assert counters_are_zero()


def test_stream_k_exact_whole_rounds_only():
    # 2048 x 2048 with 64x64 tiles: 1024 tiles, whole rounds of a grid of 256, 512 or 1024 workgroups and nothing left over
    # (no part of a tile, the workspace stays untouched); with 128x128 tiles 256 tiles
    spec = synth.gemm_spec(2048, 2048, 136, dt_out="f32", epilogue=(), integer=True)
    for tile in built(0, scheduler=2):
        parity.check_exact(spec, SK(*tile), label=f"stream-K whole rounds {tile}")
    assert counters_are_zero()


@pytest.mark.parametrize("K", [1024, 960])
def test_stream_k_exact_whole_rounds_and_a_few_tiles_left(K):
    # 66 x 16 tiles of 64x64 (33 x 8 of 128x128): whole rounds of any grid of 256, 512 or 1024 workgroups and 32 (8)
    # tiles left over, whose k steps are cut into short runs.  K = 1024: the runs divide a tile's 16 k steps and are
    # dealt k range by k range; K = 960: 15 k steps, runs of two straddle tiles and are dealt tile by tile.
    spec = synth.gemm_spec(4224, 1024, K, dt_out="f32", epilogue=(), integer=True)
    for tile in built(0, scheduler=2):
        parity.check_exact(spec, SK(*tile), label=f"stream-K rounds + rest, K={K} {tile}")
    assert counters_are_zero()


def test_stream_k_floating_point_with_epilogue_and_table_choice():
    spec = synth.gemm_spec(1100, 900, 1544, epilogue=("bias", "gelu_erf", "aux_load"))
    for tile in built(0, scheduler=2):
        parity.check(spec, SK(*tile), label=f"stream-K bias+gelu+aux_load {tile}")
    parity.check(spec, SK(), label="stream-K, the library's tile")
    assert counters_are_zero()


def test_stream_k_is_bit_identical_from_run_to_run():
    # the parts of a tile are added in k order whichever workgroup arrives last: 12 runs on one workspace, one result
    spec = synth.gemm_spec(520, 392, 4104, epilogue=("bias", "relu"))
    w = DeviceWorkload(spec)
    tile = built(0, scheduler=2)[0]
    w.run(tune=SK(*tile))
    ref = w.result_bits().copy()
    for _ in range(12):
        w.D.fill_(0x7FC1)
        w.run(tune=SK(*tile))
        assert np.array_equal(w.result_bits(), ref)
    assert counters_are_zero()


def test_stream_k_workspace_contract_and_rejections():
    spec = synth.gemm_spec(200, 136, 1992, dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    tile = (64, 64, 64, 4)
    need, parts = ucl.ucl_workspace_size("gemm", "bf16", "f32", SK(*tile), **w._problem_kwargs())
    assert need > WORKSPACE_COUNTER_BYTES and parts >= 2
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=Tuning(*tile, scheduler="stream_k"))
    assert e.value.status == "UCL_ERR_WORKSPACE" and str(need) in e.value.message
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=SK(*tile, nbytes=need - 1))
    assert e.value.status == "UCL_ERR_WORKSPACE"
    w.run(tune=SK(*tile, nbytes=need))                       # exactly enough
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
    ws = workspace()
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=Tuning(*tile, scheduler="stream_k", split_k="serial", slices=2, workspace=ws.data_ptr(), workspace_bytes=ws.numel()))
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=SK(256, 256, 64, 2))                         # built, but not with this scheduler
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    g = DeviceWorkload(synth.grouped_spec([64, 64], 64, 256, dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        g.run(tune=SK())
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    r = DeviceWorkload(synth.gemm_spec(256, 256, 256, b_layout="row", dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        r.run(tune=SK())
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    assert counters_are_zero()
