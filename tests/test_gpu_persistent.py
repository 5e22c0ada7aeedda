"""GPU parity of the persistent tile scheduler (`.with_scheduler(tile=persistent)`): the grid holds one
workgroup per CU slot and every workgroup walks the tile order with a stride of the grid size.  Exact on
integer inputs for every variant built with it, on problems with fewer tiles than slots, with several
tiles per workgroup and a ragged last round; floating point with fused epilogues against the oracle;
bit-identical to the default scheduler; unsupported combinations rejected."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning
from paper_2603_29010_amd.workload import DeviceWorkload

import parity
from test_gpu_parity import built

pytestmark = pytest.mark.gpu


def P(*tile):
    return Tuning(*tile, scheduler="persistent")


def test_persistent_variants_are_listed():
    assert built(0, scheduler=1) and built(0, f16=1, scheduler=1) and built(1, scheduler=1)
    for t in built(0, scheduler=1) + built(1, scheduler=1):
        assert t[0] <= 128 and t[1] <= 128


@pytest.mark.parametrize("tile,dt", [(t, "bf16") for t in built(0, scheduler=1)] + [(t, "f16") for t in built(0, f16=1, scheduler=1)])
def test_persistent_gemm_exact_few_tiles(tile, dt):
    # fewer tiles than CU slots: every workgroup runs its loop once; ragged M, N and a K tail
    spec = synth.gemm_spec(328, 264, 200, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, P(*tile), label=f"persistent {tile}")


@pytest.mark.parametrize("tile,dt", [(t, "bf16") for t in built(0, scheduler=1)] + [(t, "f16") for t in built(0, f16=1, scheduler=1)])
def test_persistent_gemm_exact_many_tiles(tile, dt):
    # 64x64 tiles: 58 x 57 = 3306 tiles over at most 256 x 8 slots, 128x128: 29 x 29 = 841 over at most 768:
    # several rounds per workgroup, the last one ragged; M, N not multiples of the tile
    spec = synth.gemm_spec(3700, 3600, 72, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, P(*tile), label=f"persistent many tiles {tile}")


@pytest.mark.parametrize("tile", built(0, f16=1, scheduler=1))
def test_persistent_batched_exact(tile):
    # tiles of several batches in one workgroup's walk: 40 batches x 3 x 2 (or 6 x 3) tiles
    spec = synth.batched_spec(40, 328, 136, 136, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, P(*tile), label=f"persistent batched {tile}")


@pytest.mark.parametrize("tile", built(1, scheduler=1))
def test_persistent_grouped_exact(tile):
    # empty groups, ragged groups, groups of many tiles: the walk crosses group boundaries
    M_g = [0, 700, 64, 1, 0, 2000, 130, 3000, 5, 0, 1500, 257]
    spec = synth.grouped_spec(M_g, 520, 136, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, P(*tile), label=f"persistent grouped {tile}")


def test_persistent_floating_point_with_epilogue():
    spec = synth.gemm_spec(2100, 1900, 520, epilogue=("bias", "gelu_erf", "aux_load"))
    for tile in built(0, scheduler=1):
        parity.check(spec, P(*tile), label=f"persistent bias+gelu+aux_load {tile}")
    spec = synth.grouped_spec([300, 0, 1100, 77], 384, 264, epilogue=("silu",))
    for tile in built(1, scheduler=1):
        parity.check(spec, P(*tile), label=f"persistent grouped silu {tile}")


def test_persistent_matches_default_bit_for_bit():
    spec = synth.gemm_spec(3000, 2900, 264, epilogue=("bias", "relu"))
    w = DeviceWorkload(spec)
    for tile in built(0, scheduler=1):
        w.run(tune=Tuning(*tile))
        ref = w.result_bits().copy()
        w.D.fill_(0x7FC1)
        w.run(tune=P(*tile))
        assert np.array_equal(w.result_bits(), ref), tile


def test_persistent_selection_and_rejections():
    w = DeviceWorkload(synth.gemm_spec(1024, 1024, 256, dt_out="f32", epilogue=(), integer=True))
    w.run(tune=Tuning(scheduler="persistent"))                  # the library chooses among the persistent variants
    assert np.array_equal(w.result(), parity.orc_run.run(w.spec))
    with pytest.raises(ucl.UclError) as e:
        w.run(tune=P(256, 256, 64, 2))                          # built, but not with the persistent scheduler
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    c = DeviceWorkload(synth.conv_spec(2, 8, 8, 64, 64, 3, 3, dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        c.run(tune=Tuning(scheduler="persistent"))
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
    r = DeviceWorkload(synth.gemm_spec(256, 256, 256, b_layout="row", dt_out="f32", epilogue=(), integer=True))
    with pytest.raises(ucl.UclError) as e:
        r.run(tune=Tuning(scheduler="persistent"))
    assert e.value.status == "UCL_ERR_UNSUPPORTED"
