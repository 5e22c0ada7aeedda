"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle, element by element."""
import math

import numpy as np
import pytest

from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning

import parity

pytestmark = pytest.mark.gpu


import paper_2603_29010_amd as ucl


def T(tm, tn, tk, st, raster=0, iterator=0):
    return Tuning(tm, tn, tk, st, raster, iterator)


ANALYTIC, PATCH = 1, 2      # ucl_conv_iterator


def built(mode, f16=0, la=None, lb=0, dt=None, scheduler=0, patch_c=None):
    """(tile_m, tile_n, tile_k, stages) of every kernel variant built for a problem class and
    tile scheduler (0: one workgroup per tile, 1: persistent); resident-patch variants (la 3): those for
    pixels of `patch_c` channels (default: 64 for fprop, 128 for dgrad)."""
    la = (2 if mode == 2 else 0) if la is None else la
    dt = ("f16" if f16 else "bf16") if dt is None else dt
    pc = 0 if la != 3 else patch_c if patch_c is not None else (64 if mode == 2 else 128)
    out = []
    for i in range(ucl.ucl_num_variants()):
        v = ucl.ucl_variant(i)
        if (v["mode"], v["dt"], v["la"], v["lb"], v["scheduler"], v["patch_channels"]) == (mode, dt, la, lb, scheduler, pc):
            out.append((v["tile_m"], v["tile_n"], v["tile_k"], v["stages"]))
    assert out
    return out


KK_TILES = built(0)
KK_TILES_F16 = built(0, f16=1)


# ---------------------------------------------------------------- exact (integer) indexing tests

@pytest.mark.parametrize("tile,dt", [(t, "bf16") for t in KK_TILES] + [(t, "f16") for t in KK_TILES_F16])
def test_gemm_exact_every_tile(tile, dt):
    # ragged in M and N, K tail (K = 200 = 3*64 + 8), several tiles in each direction
    spec = synth.gemm_spec(328, 264, 200, dt_in=dt, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, T(*tile), label=f"tile{tile}")


@pytest.mark.parametrize("K", [8, 40, 96, 160, 416])
def test_gemm_exact_short_k_every_tile(K):
    # K shorter than a k-tile, fewer k-tiles than pipeline stages, odd numbers of k-tiles (the loop
    # works in units of two k-tiles where a k-tile is one MFMA k-step), K tails of 8 and 32
    spec = synth.gemm_spec(264, 136, K, dt_out="f32", epilogue=(), integer=True)
    for tile in KK_TILES:
        parity.check_exact(spec, T(*tile), label=f"K{K} tile{tile}")


@pytest.mark.parametrize("a_layout,b_layout", [("row", "row"), ("col", "col"), ("col", "row")])
@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_gemm_exact_transposed_layouts(a_layout, b_layout, dt):
    spec = synth.gemm_spec(200, 136, 72, dt_in=dt, dt_out="f32", a_layout=a_layout, b_layout=b_layout, epilogue=(),
                           integer=True)
    for tile in built(0, f16=int(dt == "f16"), la=int(a_layout == "col"), lb=int(b_layout == "row")):
        parity.check_exact(spec, T(*tile), label=f"{a_layout}/{b_layout}{tile}")


# A row-major, B row-major (contiguous along N): B is copied row by row into LDS and read through the
# LDS transpose read.  Every such variant, exact: several tiles in M and N, a K tail inside a k-tile,
# K shorter than one k-tile, ragged N (multiple of 8 only), batches, a leading stride wider than N.
@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_gemm_exact_n_contiguous_b_direct(dt):
    f16 = int(dt == "f16")
    for tile in built(0, f16=f16, la=0, lb=4):
        for (M, N, K) in ((328, 264, 200), (72, 520, 40), (260, 136, 8), (520, 392, 416)):
            spec = synth.gemm_spec(M, N, K, dt_in=dt, dt_out="f32", a_layout="row", b_layout="row", epilogue=(), integer=True)
            parity.check_exact(spec, T(*tile), label=f"row/row {tile} {M}x{N}x{K}")
    spec = synth.gemm_spec(520, 392, 264, dt_in=dt, a_layout="row", b_layout="row", epilogue=("bias", "gelu_tanh"))
    for tile in built(0, f16=f16, la=0, lb=4):
        parity.check(spec, T(*tile), label=f"row/row fp {tile}")
    parity.check(spec, None, label="row/row table choice")


# A column-major (contiguous along M) copied the same way, with B contiguous along K or along N.
@pytest.mark.parametrize("b_layout", ["col", "row"])
@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_gemm_exact_m_contiguous_a_direct(dt, b_layout):
    f16 = int(dt == "f16")
    lb = 4 if b_layout == "row" else 0
    for tile in built(0, f16=f16, la=5, lb=lb):
        for (M, N, K) in ((328, 264, 200), (72, 520, 40), (264, 136, 8), (520, 392, 416)):
            spec = synth.gemm_spec(M, N, K, dt_in=dt, dt_out="f32", a_layout="col", b_layout=b_layout, epilogue=(), integer=True)
            parity.check_exact(spec, T(*tile), label=f"col/{b_layout} {tile} {M}x{N}x{K}")
    spec = synth.gemm_spec(520, 392, 264, dt_in=dt, a_layout="col", b_layout=b_layout, epilogue=("bias", "gelu_tanh"))
    for tile in built(0, f16=f16, la=5, lb=lb):
        parity.check(spec, T(*tile), label=f"col/{b_layout} fp {tile}")
    parity.check(spec, None, label=f"col/{b_layout} table choice")
    if b_layout == "row":
        # neither operand is contiguous along K: K need not be a multiple of 8
        for K in (3, 20, 45):
            spec = synth.gemm_spec(136, 72, K, dt_in=dt, dt_out="f32", a_layout="col", b_layout="row", epilogue=(), integer=True)
            for tile in built(0, f16=f16, la=5, lb=4):
                parity.check_exact(spec, T(*tile), label=f"col/row K={K} {tile}")


@pytest.mark.parametrize("shape", [(1, 8, 8), (8, 1, 8), (7, 5, 16), (64, 64, 64), (65, 63, 64), (1, 1, 8)])
def test_gemm_exact_degenerate_shapes(shape):
    M, N, K = shape
    spec = synth.gemm_spec(M, N, K, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, label=str(shape))


def test_gemm_exact_bf16_output_and_odd_n():
    # N = 77 forces the scalar-store path for the ragged last columns; |values| small enough for bf16
    spec = synth.gemm_spec(96, 77, 16, dt_out="bf16", epilogue=(), integer=True)
    parity.check_exact(spec)


@pytest.mark.parametrize("raster", [1, 2, 8, 16])
def test_gemm_exact_raster_orders(raster):
    spec = synth.gemm_spec(640, 448, 64, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec, T(64, 64, 32, 3, raster), label=f"raster{raster}")


def test_batched_exact():
    spec = synth.batched_spec(5, 136, 72, 24, dt_out="f32", epilogue=(), integer=True)
    parity.check_exact(spec)
    for tile in KK_TILES_F16:
        parity.check_exact(spec, T(*tile), label=f"batched{tile}")


@pytest.mark.parametrize("a_layout,b_layout", [("row", "row"), ("col", "col"), ("col", "row")])
def test_batched_exact_directly_copied_layouts(a_layout, b_layout):
    # batches advance the directly copied operands too (P.V-like: B stored [b, K, N])
    la, lb = (5 if a_layout == "col" else 0), (4 if b_layout == "row" else 0)
    spec = synth.batched_spec(5, 136, 200, 72, dt_in="bf16", dt_out="f32", epilogue=(), integer=True,
                              a_layout=a_layout, b_layout=b_layout)
    for tile in built(0, la=la, lb=lb):
        parity.check_exact(spec, T(*tile), label=f"batched {a_layout}/{b_layout} {tile}")
    spec = synth.batched_spec(3, 264, 136, 200, dt_in="f16", dt_out="f16", a_layout=a_layout, b_layout=b_layout)
    parity.check(spec, None, label=f"batched {a_layout}/{b_layout} fp")


def test_grouped_exact_ragged_offsets():
    M_g = [64, 0, 200, 8, 321, 0, 128, 1]
    spec = synth.grouped_spec(M_g, 136, 72, dt_out="f32", epilogue=(), integer=True)
    for tile in built(1):
        parity.check_exact(spec, T(*tile), label=f"grouped{tile}")


def test_grouped_row_major_b():
    # expert weights stored [K, N]: ragged groups, empty groups, a K tail inside a k-tile
    M_g = [64, 0, 200, 8, 321, 0, 128, 1]
    spec = synth.grouped_spec(M_g, 136, 72, dt_out="f32", epilogue=(), integer=True, b_layout="row")
    for tile in built(1, lb=4):
        parity.check_exact(spec, T(*tile), label=f"grouped row-major B {tile}")
    spec = synth.grouped_spec([200, 72, 0, 333], 264, 200, epilogue=("silu",), b_layout="row")
    for tile in built(1, lb=4):
        parity.check(spec, T(*tile), label=f"grouped row-major B fp {tile}")
    parity.check(spec, None, label="grouped row-major B table choice")
    spec16 = synth.grouped_spec([200, 72, 0, 333], 264, 200, dt_in="f16", dt_out="f16", epilogue=("silu",), b_layout="row")
    for tile in built(1, f16=1, lb=4):
        parity.check(spec16, T(*tile), label=f"grouped f16 row-major B {tile}")


# Per-group epilogue tensors through device pointer tables: every group has its own bias row, its
# slice of the packed residual and of the packed per-row vector.  Exact on integers over every grouped
# variant and both B layouts (fused fast form, fused element-predicated form via a ragged N, and
# interpreted chains), then floating point through explicit variants and the table's choice.
GROUPED_TENSOR_CHAINS = [
    ("bias",),
    ("bias", "aux_load"),
    ("per_row_scale", "bias"),
    ("column_broadcast", ("aux_load", 2.0), "row_broadcast"),
]


@pytest.mark.parametrize("b_layout", ["col", "row"])
@pytest.mark.parametrize("chain", GROUPED_TENSOR_CHAINS, ids=lambda c: "-".join(s if isinstance(s, str) else s[0] for s in c))
def test_grouped_exact_per_group_epilogue_tensors(chain, b_layout):
    M_g = [64, 0, 200, 8, 321, 0, 128, 1]
    spec = synth.grouped_spec(M_g, 136, 72, dt_out="f32", epilogue=chain, integer=True, b_layout=b_layout)
    for tile in built(1, lb=4 if b_layout == "row" else 0):
        parity.check_exact(spec, T(*tile), label=f"grouped {chain} {b_layout} {tile}")
    parity.check_exact(spec, None, label=f"grouped {chain} {b_layout} table choice")


def test_grouped_exact_per_group_tensors_ragged_n():
    # N % 8 != 0: D rows and the residual are accessed element by element, bias rows stay 16-byte
    # aligned; group sizes are multiples of 8 so that every per-group base pointer is aligned
    M_g = [64, 0, 200, 8, 328, 128]
    for chain in (("bias", "aux_load", "relu"), ("per_row_scale", "bias", "aux_load")):
        for dt_out in ("f32", "bf16"):
            spec = synth.grouped_spec(M_g, 77, 24, dt_out=dt_out, epilogue=chain, integer=True)
            for tile in built(1):
                parity.check_exact(spec, T(*tile), label=f"grouped N=77 {chain} {dt_out} {tile}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_grouped_parity_per_group_epilogue_tensors(dt):
    f16 = int(dt == "f16")
    for chain in (("bias", "aux_load", "relu"), ("bias", "gelu_tanh"), ("per_row_scale", "per_col_scale", "silu"),
                  (("scale", 0.5), "column_broadcast", ("aux_load", -0.5), "tanh")):
        for b_layout, lb in (("col", 0), ("row", 4)):
            spec = synth.grouped_spec([192, 64, 0, 448, 129], 264, 136, dt_in=dt, dt_out=dt, epilogue=chain, b_layout=b_layout)
            for tile in built(1, f16=f16, lb=lb):
                parity.check(spec, T(*tile), label=f"grouped {dt} {chain} {b_layout} {tile}")
            parity.check(spec, None, label=f"grouped {dt} {chain} {b_layout} table choice")


@pytest.mark.parametrize("geom", [
    dict(Nb=2, H=9, W=7, C=16, Ko=24, R=3, S=3, pad=(1, 1)),
    dict(Nb=1, H=12, W=10, C=8, Ko=8, R=5, S=3, pad=(2, 0), stride=(2, 1)),
    dict(Nb=3, H=8, W=8, C=24, Ko=40, R=3, S=3, pad=(2, 2), dil=(2, 2)),
    dict(Nb=2, H=6, W=6, C=64, Ko=16, R=1, S=1, pad=(0, 0)),
    dict(Nb=1, H=1, W=40, C=8, Ko=8, R=1, S=5, pad=(0, 2)),           # conv1d as H = 1
    dict(Nb=2, H=7, W=9, C=72, Ko=136, R=3, S=2, pad=(1, 1), stride=(2, 3)),
])
def test_conv_exact_every_halo_position(geom):
    spec = synth.conv_spec(dt_out="f32", epilogue=(), integer=True, **geom)
    for tile in built(2):
        parity.check_exact(spec, T(*tile, iterator=ANALYTIC), label=f"conv{tile}")


# 3x3 / stride 1 / pad 1 / 64 channels: geometries the resident-patch kernels accept.  Tiles of 256
# pixels that start and end mid-row and cross image boundaries, one-pixel-wide and one-row-high
# images, the widest row the patch holds, ragged M and N tails; the per-tap gather runs beside it.
@pytest.mark.parametrize("geom", [
    dict(Nb=3, H=13, W=11, Ko=72),
    dict(Nb=2, H=20, W=58, Ko=128),
    dict(Nb=5, H=1, W=1, Ko=8),
    dict(Nb=2, H=9, W=1, Ko=24),
    dict(Nb=2, H=1, W=37, Ko=136),
    dict(Nb=7, H=6, W=6, Ko=16),
    dict(Nb=1, H=56, W=56, Ko=128),
])
def test_conv_patch_iterator_exact(geom):
    spec = synth.conv_spec(C=64, R=3, S=3, dt_out="f32", epilogue=(), integer=True, **geom)
    for tile in built(2, la=3):
        parity.check_exact(spec, T(*tile, iterator=PATCH), label=f"conv patch {tile}")
    parity.check_exact(spec, T(256, 128, 32, 3, iterator=ANALYTIC), label="conv gather")
    parity.check_exact(spec, None, label="conv table choice")


@pytest.mark.parametrize("geom", [
    dict(Nb=3, H=13, W=11, Ko=72),
    dict(Nb=2, H=20, W=58, Ko=64),
    dict(Nb=2, H=9, W=1, Ko=24),
    dict(Nb=2, H=1, W=37, Ko=136),
    dict(Nb=4, H=28, W=28, Ko=128),
])
def test_conv_patch_iterator_exact_128_channels(geom):
    # pixels of 128 channels: patch rows of 256 bytes, four k-tiles per tap
    spec = synth.conv_spec(C=128, R=3, S=3, dt_out="f32", epilogue=(), integer=True, **geom)
    for tile in built(2, la=3, patch_c=128):
        parity.check_exact(spec, T(*tile, iterator=PATCH), label=f"conv patch, 128 channels {tile}")
    parity.check_exact(spec, T(256, 128, 32, 3, iterator=ANALYTIC), label="conv gather")
    parity.check_exact(spec, None, label="conv table choice")
    spec16 = synth.conv_spec(C=128, R=3, S=3, dt_in="f16", dt_out="f16", epilogue=("bias", "relu"), **geom)
    for tile in built(2, f16=1, la=3, patch_c=128):
        parity.check(spec16, T(*tile, iterator=PATCH), label=f"conv f16 patch, 128 channels {tile}")


def test_conv_patch_iterator_refuses_other_geometries():
    for kw in (dict(C=32), dict(R=1, S=1, pad=(0, 0)), dict(stride=(2, 2)), dict(dil=(2, 2), pad=(2, 2)), dict(W=59), dict(pad=(0, 0))):
        g = dict(Nb=1, H=8, W=8, C=64, Ko=16, R=3, S=3)
        g.update(kw)
        spec = synth.conv_spec(dt_out="f32", epilogue=(), integer=True, **g)
        with pytest.raises(ucl.UclError) as e:
            parity.gpu_result(spec, T(0, 0, 0, 0, iterator=PATCH))
        assert e.value.status == "UCL_ERR_UNSUPPORTED" and "fixed_stride_dilation" in str(e.value)
        parity.check_exact(spec, None, label=f"conv {kw}")


# ---------------------------------------------------------------- floating-point parity

@pytest.mark.parametrize("tile", KK_TILES)
def test_gemm_parity_every_tile(tile):
    spec = synth.gemm_spec(520, 392, 264, epilogue=("bias", "gelu_tanh"))
    parity.check(spec, T(*tile), label=f"tile{tile}")


@pytest.mark.parametrize("tile", KK_TILES)
def test_gemm_parity_every_tile_fp32_output(tile):
    # fp32 output without a residual: wide wave tiles hand each lane two 4-column groups a row apart
    # (bias index and store offsets follow); the same chain with a residual keeps 8 consecutive columns
    spec = synth.gemm_spec(520, 392, 264, dt_out="f32", epilogue=(("scale", 0.5), "bias", "gelu_tanh"))
    parity.check(spec, T(*tile), label=f"f32 out tile{tile}")
    bias, dt = spec["tensors"]["bias11"]
    spec["tensors"]["bias11"] = (synth.to_bits(synth.bits_to_f64(bias, dt), "bf16"), "bf16")     # 16-bit bias, fp32 output
    parity.check(spec, T(*tile), label=f"f32 out, bf16 bias, tile{tile}")
    spec = synth.gemm_spec(520, 392, 264, dt_out="f32", epilogue=("bias", "aux_load", "relu"))
    parity.check(spec, T(*tile), label=f"f32 out with residual tile{tile}")


ALL_CHAINS = [
    ("bias", "relu"),
    ("bias", "gelu_tanh"),
    ("gelu_erf",),
    ("silu",),
    (("scale", 0.125), "sigmoid"),
    ("tanh",),
    ("mish",),
    ("hardswish",),
    (("leaky_relu", 0.1),),
    (("elu", 1.5),),
    ("bias", ("clamp", -0.5, 0.75)),
    ("per_row_scale", "per_col_scale"),
    ("row_broadcast", "column_broadcast", "relu"),
    (("scale", 2.0), ("aux_load", -0.5), "relu"),
    ("bias", "aux_load", "relu", ("scale", 3.0), "tanh", ("clamp", 0.0, 6.0), "silu", "hardswish"),
]


@pytest.mark.parametrize("chain", ALL_CHAINS, ids=lambda c: "-".join(s if isinstance(s, str) else s[0] for s in c))
@pytest.mark.parametrize("dt_out", ["bf16", "f32"])
def test_epilogue_vocabulary(chain, dt_out):
    spec = synth.gemm_spec(136, 200, 128, dt_out=dt_out, dist="normal", scale=0.25, epilogue=chain)
    parity.check(spec, label=str(chain))


def test_aux_store_captures_mid_chain_value():
    import oracle
    from paper_2603_29010_amd.workload import DeviceWorkload
    spec = synth.gemm_spec(72, 136, 64, dt_out="bf16", epilogue=("bias", "relu"))
    spec["epilogue"].insert(1, ("aux_store", "pre_act", "f32"))
    w = DeviceWorkload(spec)
    w.run()
    got = w.result()
    pre = w.aux_result("pre_act")
    base = dict(spec)
    base["epilogue"] = [spec["epilogue"][0]]
    ref_pre, s1 = parity.oracle_result(base)
    parity.compare(pre, ref_pre, s1, dict(base, dt_out="f32"), "aux_store")
    base["epilogue"] = [spec["epilogue"][0], spec["epilogue"][2]]
    ref, s2 = parity.oracle_result(base)
    parity.compare(got, ref, s2, base, "after aux_store")


@pytest.mark.parametrize("dt_in,dt_out", [("f16", "f16"), ("f16", "f32"), ("bf16", "f16")])
def test_gemm_dtype_combinations(dt_in, dt_out):
    spec = synth.gemm_spec(200, 136, 136, dt_in=dt_in, dt_out=dt_out, epilogue=("bias", "silu"))
    parity.check(spec)


def test_batched_parity_with_residual():
    spec = synth.batched_spec(3, 136, 200, 72, dt_out="f16", epilogue=[("scale", 0.5), "aux_load", "relu"])
    parity.check(spec)


def test_grouped_parity_silu():
    spec = synth.grouped_spec([192, 64, 0, 448, 128], 264, 136)
    for tile in built(1):
        parity.check(spec, T(*tile), label=f"grouped{tile}")
    spec16 = synth.grouped_spec([192, 64, 0, 448, 128], 264, 136, dt_in="f16", dt_out="f16")
    for tile in built(1, f16=1):
        parity.check(spec16, T(*tile), label=f"grouped f16 {tile}")


def test_conv_parity_bias_residual_relu():
    spec = synth.conv_spec(3, 14, 14, 64, 128, 3, 3)
    for tile in built(2):
        parity.check(spec, T(*tile, iterator=ANALYTIC), label=f"conv{tile}")
    for tile in built(2, la=3):
        parity.check(spec, T(*tile, iterator=PATCH), label=f"conv patch {tile}")
    spec16 = synth.conv_spec(3, 14, 14, 64, 128, 3, 3, dt_in="f16", dt_out="f32")
    for tile in built(2, f16=1):
        parity.check(spec16, T(*tile, iterator=ANALYTIC), label=f"conv f16 {tile}")
    for tile in built(2, f16=1, la=3):
        parity.check(spec16, T(*tile, iterator=PATCH), label=f"conv f16 patch {tile}")


@pytest.mark.parametrize("geom", [dict(Nb=3, H=13, W=11, Ko=72), dict(Nb=2, H=20, W=58, Ko=136), dict(Nb=5, H=1, W=1, Ko=8),
                                  dict(Nb=4, H=31, W=29, Ko=128)])
@pytest.mark.parametrize("dt_out", ["bf16", "f32"])
def test_conv_patch_residual_ragged(geom, dt_out):
    # the patch kernels touch the tile's 16-bit residual lines during the mainloop (a prefetch into L2): tiles whose last
    # rows and columns do not exist, a residual row shorter than one line, an fp32 residual (no prefetch)
    spec = synth.conv_spec(C=64, R=3, S=3, dt_out=dt_out, **geom)
    for tile in built(2, la=3):
        parity.check(spec, T(*tile, iterator=PATCH), label=f"conv patch residual {tile}")


# ---------------------------------------------------------------- the benchmark configurations

def test_config1_full():
    parity.check(synth.config(1), label="config1")


def test_config2_shrunk_and_default_selection():
    parity.check(synth.config(2, shrink=8), label="config2/8")


def test_config3_shrunk():
    parity.check(synth.config(3, shrink=16), label="config3/16")


def test_config4_shrunk():
    parity.check(synth.config(4, shrink=8), label="config4/8")


def test_config5_shrunk():
    parity.check(synth.config(5, shrink=16), label="config5/16")


# Full size, in the launch configuration bench.py times (selection table's choice), EVERY output
# element against the oracle: a wrong or unwritten tile anywhere fails.

def test_config2_full_size_every_element():
    parity.check(synth.config(2), label="config2 full")


def test_config3_full_size():
    parity.check(synth.config(3), label="config3 full")


def test_config4_full_size_every_element():
    parity.check(synth.config(4), label="config4 full")


def test_config5_full_size_every_element():
    parity.check(synth.config(5), label="config5 full")


def test_hip_graph_replays_match_eager_launch():
    """bench.py times launches recorded in a HIP graph: every replay must give the eager result.
    The library issues kernel nodes only (no memset or copy nodes); the replays are separated by
    eager work and synchronisation of the program's own."""
    import torch
    from paper_2603_29010_amd.workload import DeviceWorkload
    spec = synth.config(2, shrink=8)
    w = DeviceWorkload(spec)
    w.run()
    torch.cuda.synchronize()
    eager = w.result().copy()
    ref, absacc = parity.oracle_result(spec)
    parity.compare(eager.reshape(ref.shape), ref, absacc, spec, "eager")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        w.run()
        w.run()
    for rep in range(3):
        w.D.zero_()                       # eager work between replays; also wipes the previous result
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = w.result()
        assert np.array_equal(got, eager), f"replay {rep} differs from the eager launch"
