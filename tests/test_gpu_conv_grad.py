"""GPU parity of conv2d_dgrad and conv2d_wgrad (the index maps of the two gradients on the shared
mainloop) against the fp64 oracle: exact on integer inputs over every built variant and every halo /
stride / dilation class, floating point with fused epilogues, wgrad with split-K."""
import numpy as np
import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning

import parity
from test_gpu_parity import T, built

pytestmark = pytest.mark.gpu

GEOMS = [
    dict(Nb=2, H=9, W=7, C=16, Ko=24, R=3, S=3, pad=(1, 1)),
    dict(Nb=1, H=12, W=10, C=8, Ko=8, R=5, S=3, pad=(2, 0), stride=(2, 1)),
    dict(Nb=3, H=8, W=8, C=24, Ko=40, R=3, S=3, pad=(2, 2), dil=(2, 2)),
    dict(Nb=2, H=6, W=6, C=64, Ko=16, R=1, S=1, pad=(0, 0)),
    dict(Nb=1, H=1, W=40, C=8, Ko=8, R=1, S=5, pad=(0, 2)),              # 1-D convolution as H = 1
    dict(Nb=2, H=7, W=9, C=72, Ko=136, R=3, S=2, pad=(1, 1), stride=(2, 3)),
    dict(Nb=2, H=11, W=13, C=8, Ko=16, R=3, S=3, pad=(0, 1), stride=(3, 2), dil=(2, 1)),   # input rows the filter never reaches
    dict(Nb=5, H=14, W=14, C=32, Ko=64, R=3, S=3, pad=(1, 1)),             # several tiles of rows / a deep K
]
IDS = [f"{g['H']}x{g['W']}x{g['C']}-{g['Ko']}-{g['R']}x{g['S']}" for g in GEOMS]


@pytest.mark.parametrize("geom", GEOMS, ids=IDS)
def test_dgrad_exact_every_variant(geom):
    spec = synth.conv_grad_spec("dgrad", dt_out="f32", integer=True, **geom)
    for tile in built(3, la=2, lb=4):
        parity.check_exact(spec, T(*tile), label=f"dgrad {tile}")
    parity.check_exact(spec, None, label="dgrad table choice")


# 3x3 / stride 1 / pad 1 / 128 output channels: geometries the resident-patch data-gradient kernels accept (the
# output gradient of a tile held in LDS, taps mirrored).  Tiles that start and end mid-row and cross image
# boundaries, one-pixel-wide and one-row-high images, the widest row the patch holds, ragged M and C tails;
# the per-tap gather runs beside it.
ANALYTIC, PATCH = 1, 2      # ucl_conv_iterator


@pytest.mark.parametrize("geom", [
    dict(Nb=3, H=13, W=11, C=72),
    dict(Nb=2, H=20, W=58, C=64),
    dict(Nb=5, H=1, W=1, C=8),
    dict(Nb=2, H=9, W=1, C=24),
    dict(Nb=2, H=1, W=37, C=136),
    dict(Nb=7, H=6, W=6, C=16),
    dict(Nb=1, H=56, W=56, C=64),
])
def test_dgrad_patch_iterator_exact(geom):
    spec = synth.conv_grad_spec("dgrad", Ko=128, R=3, S=3, pad=(1, 1), dt_out="f32", integer=True, **geom)
    for tile in built(3, la=3, lb=4):
        parity.check_exact(spec, T(*tile, iterator=PATCH), label=f"dgrad patch {tile}")
    parity.check_exact(spec, T(256, 64, 32, 4, iterator=ANALYTIC), label="dgrad gather")
    parity.check_exact(spec, None, label="dgrad table choice")


@pytest.mark.parametrize("geom", [
    dict(Nb=3, H=13, W=11, C=72),
    dict(Nb=2, H=20, W=58, C=128),
    dict(Nb=2, H=9, W=1, C=24),
    dict(Nb=2, H=1, W=37, C=136),
    dict(Nb=2, H=56, W=56, C=64),
])
def test_dgrad_patch_iterator_exact_64_channels(geom):
    # an output gradient of 64 channels: patch rows of 128 bytes, two k-tiles per tap
    spec = synth.conv_grad_spec("dgrad", Ko=64, R=3, S=3, pad=(1, 1), dt_out="f32", integer=True, **geom)
    for tile in built(3, la=3, lb=4, patch_c=64):
        parity.check_exact(spec, T(*tile, iterator=PATCH), label=f"dgrad patch, 64 channels {tile}")
    parity.check_exact(spec, T(256, 64, 32, 4, iterator=ANALYTIC), label="dgrad gather")
    parity.check_exact(spec, None, label="dgrad table choice")
    spec16 = synth.conv_grad_spec("dgrad", Ko=64, R=3, S=3, pad=(1, 1), dt_in="f16", dt_out="f16", epilogue=("bias", "relu"), **geom)
    for tile in built(3, f16=1, la=3, lb=4, patch_c=64):
        parity.check(spec16, T(*tile, iterator=PATCH), label=f"dgrad f16 patch, 64 channels {tile}")


def test_dgrad_patch_iterator_parity_and_refusals():
    g = dict(Nb=2, H=20, W=17, C=72, Ko=128, R=3, S=3, pad=(1, 1))
    spec = synth.conv_grad_spec("dgrad", epilogue=("bias", "aux_load", "relu"), **g)
    for tile in built(3, la=3, lb=4):
        parity.check(spec, T(*tile, iterator=PATCH), label=f"dgrad patch epilogue {tile}")
    spec16 = synth.conv_grad_spec("dgrad", dt_in="f16", dt_out="f16", epilogue=("gelu_tanh",), **g)
    for tile in built(3, f16=1, la=3, lb=4):
        parity.check(spec16, T(*tile, iterator=PATCH), label=f"dgrad f16 patch {tile}")
    for kw in (dict(Ko=32), dict(R=1, S=1, pad=(0, 0)), dict(stride=(2, 2)), dict(dil=(2, 2), pad=(2, 2)), dict(W=59), dict(pad=(0, 0))):
        gg = dict(Nb=1, H=8, W=8, C=16, Ko=128, R=3, S=3, pad=(1, 1))
        gg.update(kw)
        bad = synth.conv_grad_spec("dgrad", dt_out="f32", integer=True, **gg)
        with pytest.raises(ucl.UclError) as e:
            parity.gpu_result(bad, T(0, 0, 0, 0, iterator=PATCH))
        assert e.value.status == "UCL_ERR_UNSUPPORTED" and "fixed_stride_dilation" in str(e.value)
        parity.check_exact(bad, None, label=f"dgrad {kw}")


@pytest.mark.parametrize("geom", GEOMS, ids=IDS)
def test_wgrad_exact_every_variant(geom):
    spec = synth.conv_grad_spec("wgrad", dt_out="f32", integer=True, **geom)
    for tile in built(4, la=5, lb=4):
        parity.check_exact(spec, T(*tile), label=f"wgrad {tile}")
    parity.check_exact(spec, None, label="wgrad table choice")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_grads_exact_both_input_types(dt):
    g = GEOMS[0]
    f16 = int(dt == "f16")
    spec = synth.conv_grad_spec("dgrad", dt_in=dt, dt_out="f32", integer=True, **g)
    for tile in built(3, f16=f16, la=2, lb=4):
        parity.check_exact(spec, T(*tile), label=f"dgrad {dt} {tile}")
    spec = synth.conv_grad_spec("wgrad", dt_in=dt, dt_out="f32", integer=True, **g)
    for tile in built(4, f16=f16, la=5, lb=4):
        parity.check_exact(spec, T(*tile), label=f"wgrad {dt} {tile}")


def test_grads_parity_with_epilogues():
    g = dict(Nb=3, H=14, W=14, C=64, Ko=128, R=3, S=3, pad=(1, 1))
    spec = synth.conv_grad_spec("dgrad", epilogue=("bias", "aux_load", "relu"), **g)
    for tile in built(3, la=2, lb=4):
        parity.check(spec, T(*tile), label=f"dgrad fp {tile}")
    parity.check(spec, None, label="dgrad fp table choice")
    spec = synth.conv_grad_spec("wgrad", dt_out="f32", epilogue=(("scale", 0.5), "per_row_scale"), **g)
    for tile in built(4, la=5, lb=4):
        parity.check(spec, T(*tile), label=f"wgrad fp {tile}")
    spec16 = synth.conv_grad_spec("wgrad", dt_in="f16", dt_out="f16", stride=(2, 2), **g)
    parity.check(spec16, None, label="wgrad f16 strided")
    spec16 = synth.conv_grad_spec("dgrad", dt_in="f16", dt_out="f16", stride=(2, 2), epilogue=("gelu_tanh",), **g)
    parity.check(spec16, None, label="dgrad f16 strided")


@pytest.mark.parametrize("mode", ["serial", "parallel"])
def test_wgrad_split_k(mode):
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    # K = 5 * 14 * 14 = 980 output pixels: slices end in the middle of an image row
    g = dict(Nb=5, H=14, W=14, C=32, Ko=64, R=3, S=3, pad=(1, 1))
    spec = synth.conv_grad_spec("wgrad", dt_out="f32", integer=True, **g)
    for tile in built(4, la=5, lb=4):
        for slices in (2, 3, 7):
            tune = Tuning(*tile, split_k=mode, slices=slices, workspace=ws.data_ptr(), workspace_bytes=ws.numel())
            parity.check_exact(spec, tune, label=f"wgrad split-K {mode} x{slices} {tile}")
    spec = synth.conv_grad_spec("wgrad", dt_out="f32", stride=(2, 1), epilogue=(("scale", 0.25),), **g)
    tune = Tuning(split_k=mode, slices=0, workspace=ws.data_ptr(), workspace_bytes=ws.numel())
    parity.check(spec, tune, label=f"wgrad split-K {mode} auto")
    need, slices = ucl.ucl_workspace_size("conv2d_wgrad", "bf16", "f32", Tuning(split_k=mode),
                                          conv=(5, 14, 14, 32, 64, 3, 3, 1, 1, 2, 1, 1, 1))
    assert slices > 1 and need <= ws.numel()
    assert int(ws[:65536].count_nonzero().item()) == 0


def test_resnet_stage_gradients_full_size():
    # the gradients of the benchmark's convolution (32 x 56 x 56 x 64 -> 128, 3x3): sampled rows of dx, all of dw
    g = dict(Nb=32, H=56, W=56, C=64, Ko=128, R=3, S=3, pad=(1, 1))
    spec = synth.conv_grad_spec("dgrad", **g)
    rng = np.random.default_rng(7)
    rows = sorted(set(rng.integers(0, spec["M"], 300).tolist()) | {0, 55, 56 * 55, 56 * 56 - 1, spec["M"] - 1})
    parity.check(spec, rows=rows, label="dgrad 32x56x56")
    spec = synth.conv_grad_spec("wgrad", dt_out="f32", **g)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    parity.check(spec, Tuning(split_k="serial", workspace=ws.data_ptr(), workspace_bytes=ws.numel()), label="wgrad 32x56x56 split-K")
    # parallel mode (many slices, the reduction kernel stores dw itself) against serial mode with the same tile and
    # slices: the same additions in the same order, so the same bits
    from paper_2603_29010_amd.workload import DeviceWorkload
    w = DeviceWorkload(spec)
    out = {}
    for mode in ("serial", "parallel"):
        w.D.fill_(float("nan"))
        w.run(tune=Tuning(128, 128, 32, 4, split_k=mode, slices=51, workspace=ws.data_ptr(), workspace_bytes=ws.numel()))
        out[mode] = w.result_bits().copy()
    assert np.isfinite(out["parallel"]).all() and np.array_equal(out["serial"], out["parallel"])


def test_grad_validation():
    P = 4096
    with pytest.raises(ucl.UclError) as e:
        ucl.ucl_conv2d_dgrad(1, 8, 8, 8, 12, 3, 3, 1, 1, 1, 1, 1, 1, P, "bf16", P, "bf16", P, "bf16")
    assert e.value.status == "UCL_ERR_UNSUPPORTED" and "multiples of 8" in e.value.message
    with pytest.raises(ucl.UclError) as e:
        ucl.ucl_conv2d_wgrad(1, 2, 2, 8, 8, 5, 5, 0, 0, 1, 1, 1, 1, P, "bf16", P, "bf16", P, "bf16")
    assert e.value.status == "UCL_ERR_INVALID_ARG"
    with pytest.raises(ucl.UclError) as e:
        ucl.ucl_conv2d_wgrad(1, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, P, "bf16", 0, "bf16", P, "bf16")
    assert e.value.status == "UCL_ERR_INVALID_ARG"
