"""Pins for the oracle's conv2d_dgrad / conv2d_wgrad (the adjoints of conv2d_fprop with respect to
the activations and to the filter): torch fp64 autograd and conv_transpose2d on the CPU, the adjoint
identity <dy, fprop(x, w)> = <dgrad(dy, w), x> = <wgrad(dy, x), w>, delta filters, tap counts.  CPU only."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2603_29010_amd import synth


def val(a, dt):
    return synth.bits_to_f64(a, dt)


def rand_bits(shape, dt, seed, lo=-3, hi=3):
    n = int(np.prod(shape))
    return synth.to_bits(synth.randint(seed, 1, n, lo, hi) * 0.25, dt).reshape(shape)


GEOMS = [
    dict(Nb=2, H=7, W=6, C=3, Ko=4, R=3, S=3, pad=(1, 1), stride=(1, 1), dil=(1, 1)),
    dict(Nb=1, H=9, W=8, C=2, Ko=3, R=3, S=2, pad=(1, 0), stride=(2, 1), dil=(1, 1)),
    dict(Nb=2, H=8, W=9, C=2, Ko=2, R=2, S=3, pad=(2, 2), stride=(2, 3), dil=(2, 1)),
    dict(Nb=1, H=10, W=7, C=4, Ko=2, R=3, S=3, pad=(0, 2), stride=(3, 2), dil=(1, 2)),
    dict(Nb=3, H=5, W=5, C=2, Ko=5, R=1, S=1, pad=(0, 0), stride=(1, 1), dil=(1, 1)),
    dict(Nb=1, H=6, W=6, C=1, Ko=1, R=5, S=5, pad=(2, 2), stride=(1, 1), dil=(1, 1)),
]


def out_dims(g):
    P = (g["H"] + 2 * g["pad"][0] - g["dil"][0] * (g["R"] - 1) - 1) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["dil"][1] * (g["S"] - 1) - 1) // g["stride"][1] + 1
    return P, Q


def make(g, seed):
    P, Q = out_dims(g)
    x = rand_bits((g["Nb"], g["H"], g["W"], g["C"]), "bf16", seed)
    w = rand_bits((g["Ko"], g["R"], g["S"], g["C"]), "bf16", seed + 1)
    dy = rand_bits((g["Nb"], P, Q, g["Ko"]), "bf16", seed + 2)
    return x, w, dy, P, Q


def geom_args(g):
    return (g["Nb"], g["H"], g["W"], g["C"], g["Ko"], g["R"], g["S"])


def geom_kw(g):
    return dict(pad=g["pad"], stride=g["stride"], dil=g["dil"])


@pytest.mark.parametrize("g", GEOMS, ids=lambda g: "x".join(str(v) for v in (g["H"], g["W"], g["R"], g["S"])) + f"s{g['stride']}d{g['dil']}")
def test_grads_match_torch_autograd_fp64(g):
    x, w, dy, P, Q = make(g, 100)
    xt = torch.from_numpy(val(x, "bf16")).permute(0, 3, 1, 2).clone().requires_grad_(True)
    wt = torch.from_numpy(val(w, "bf16")).permute(0, 3, 1, 2).clone().requires_grad_(True)
    y = F.conv2d(xt, wt, padding=g["pad"], stride=g["stride"], dilation=g["dil"])
    assert tuple(y.shape) == (g["Nb"], g["Ko"], P, Q)
    y.backward(torch.from_numpy(val(dy, "bf16")).permute(0, 3, 1, 2))
    dx_ref = xt.grad.permute(0, 2, 3, 1).reshape(-1, g["C"]).numpy()
    dw_ref = wt.grad.permute(0, 2, 3, 1).reshape(g["Ko"], -1).numpy()
    dx = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), **geom_kw(g))
    dw = oracle.conv2d_wgrad(dy, "bf16", x, "bf16", *geom_args(g), **geom_kw(g))
    np.testing.assert_allclose(dx, dx_ref, atol=1e-10)
    np.testing.assert_allclose(dw, dw_ref, atol=1e-10)


def test_dgrad_is_the_transposed_convolution():
    g = GEOMS[1]
    x, w, dy, P, Q = make(g, 200)
    wt = torch.from_numpy(val(w, "bf16")).permute(0, 3, 1, 2)          # [Ko, C, R, S] = conv_transpose2d's layout
    gt = torch.from_numpy(val(dy, "bf16")).permute(0, 3, 1, 2)
    full = F.conv_transpose2d(gt, wt, stride=g["stride"], padding=g["pad"], dilation=g["dil"])
    # conv_transpose2d returns the smallest input size that gives (P, Q); the real input may be a few
    # rows / columns larger (the pixels the strided filter never reached get gradient zero)
    ref = torch.zeros(g["Nb"], g["C"], g["H"], g["W"], dtype=torch.float64)
    ref[:, :, :full.shape[2], :full.shape[3]] = full
    dx = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), **geom_kw(g))
    np.testing.assert_allclose(dx, ref.permute(0, 2, 3, 1).reshape(-1, g["C"]).numpy(), atol=1e-10)


@pytest.mark.parametrize("g", GEOMS[:4], ids=lambda g: f"s{g['stride']}d{g['dil']}")
def test_adjoint_identity(g):
    x, w, dy, P, Q = make(g, 300)
    y = oracle.conv2d_fprop(x, "bf16", w, "bf16", *geom_args(g), **geom_kw(g))
    dx = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), **geom_kw(g))
    dw = oracle.conv2d_wgrad(dy, "bf16", x, "bf16", *geom_args(g), **geom_kw(g))
    lhs = float(np.sum(val(dy, "bf16").reshape(y.shape) * y))
    assert lhs == pytest.approx(float(np.sum(dx * val(x, "bf16").reshape(dx.shape))), abs=1e-9)
    assert lhs == pytest.approx(float(np.sum(dw * val(w, "bf16").reshape(dw.shape))), abs=1e-9)
    assert abs(lhs) > 1.0                       # a trivial zero would satisfy the identity too


def test_delta_filters_fix_the_orientation():
    Nb, H, W, Cc = 1, 5, 6, 3
    dy = rand_bits((Nb, H, W, Cc), "bf16", 400)
    g = val(dy, "bf16")
    # centre tap, identity over channels: fprop copies, so dgrad copies too
    w = np.zeros((Cc, 3, 3, Cc))
    for k in range(Cc):
        w[k, 1, 1, k] = 1.0
    dx = oracle.conv2d_dgrad(dy, "bf16", synth.to_bits(w, "bf16"), "bf16", Nb, H, W, Cc, Cc, 3, 3, pad=(1, 1))
    assert np.array_equal(dx.reshape(g.shape), g)
    # tap (r, s) = (0, 2): y[p, q] = x[p - 1, q + 1], so dx[h, w] = dy[h + 1, w - 1] (the opposite shift)
    w = np.zeros((Cc, 3, 3, Cc))
    for k in range(Cc):
        w[k, 0, 2, k] = 1.0
    dx = oracle.conv2d_dgrad(dy, "bf16", synth.to_bits(w, "bf16"), "bf16", Nb, H, W, Cc, Cc, 3, 3, pad=(1, 1)).reshape(g.shape)
    want = np.zeros_like(g)
    want[:, :H - 1, 1:, :] = g[:, 1:, :W - 1, :]
    assert np.array_equal(dx, want)
    # wgrad with x = one-hot pixel: dw[ko, r, s, c0] = dy at the output pixel that tap (r, s) pairs with it
    x = np.zeros((Nb, H, W, Cc))
    x[0, 2, 3, 1] = 1.0
    dw = oracle.conv2d_wgrad(dy, "bf16", synth.to_bits(x, "bf16"), "bf16", Nb, H, W, Cc, Cc, 3, 3, pad=(1, 1)).reshape(Cc, 3, 3, Cc)
    for r, s in itertools.product(range(3), repeat=2):
        p, q = 2 + 1 - r, 3 + 1 - s                  # p - 1 + r = 2, q - 1 + s = 3
        assert np.array_equal(dw[:, r, s, 1], g[0, p, q, :])
        assert not dw[:, r, s, 0].any() and not dw[:, r, s, 2].any()


def test_all_ones_count_taps():
    Nb, H, W, Cc, Ko = 2, 6, 5, 2, 3
    ones = lambda *sh: synth.to_bits(np.ones(sh), "bf16")
    # 3x3, pad 1, stride 1: dx counts the output pixels a input pixel feeds (9 / 6 / 4) times Ko
    dx = oracle.conv2d_dgrad(ones(Nb, H, W, Ko), "bf16", ones(Ko, 3, 3, Cc), "bf16", Nb, H, W, Cc, Ko, 3, 3, pad=(1, 1)).reshape(Nb, H, W, Cc)
    assert dx[0, 2, 2, 0] == 9 * Ko and dx[0, 0, 2, 1] == 6 * Ko and dx[1, H - 1, W - 1, 0] == 4 * Ko
    # dw counts the output pixels whose tap (r, s) lies inside the image
    dw = oracle.conv2d_wgrad(ones(Nb, H, W, Ko), "bf16", ones(Nb, H, W, Cc), "bf16", Nb, H, W, Cc, Ko, 3, 3, pad=(1, 1)).reshape(Ko, 3, 3, Cc)
    assert dw[0, 1, 1, 0] == Nb * H * W and dw[2, 0, 1, 1] == Nb * (H - 1) * W and dw[1, 2, 0, 0] == Nb * (H - 1) * (W - 1)


def test_row_subsets_abs_sums_and_epilogue_coordinates():
    g = GEOMS[2]
    x, w, dy, P, Q = make(g, 500)
    bias_c = rand_bits((g["C"],), "f32", 501).astype(np.float32)
    dx_full, s_full = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), chain=[("bias", bias_c, "f32"), ("relu",)],
                                          want_abs=True, **geom_kw(g))
    plain = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), **geom_kw(g))
    np.testing.assert_allclose(dx_full, np.maximum(plain + bias_c[None, :].astype(np.float64), 0), atol=1e-12)
    rows = [dx_full.shape[0] - 1, 0, 5]
    sub, s_sub = oracle.conv2d_dgrad(dy, "bf16", w, "bf16", *geom_args(g), chain=[("bias", bias_c, "f32"), ("relu",)],
                                     rows=rows, want_abs=True, **geom_kw(g))
    assert np.array_equal(sub, dx_full[rows]) and np.array_equal(s_sub, s_full[rows])
    # |.| sums: the same gradients of |dy|, |w|
    abs_dx = oracle.conv2d_dgrad(synth.to_bits(np.abs(val(dy, "bf16")), "bf16"), "bf16", synth.to_bits(np.abs(val(w, "bf16")), "bf16"),
                                 "bf16", *geom_args(g), **geom_kw(g))
    np.testing.assert_allclose(s_full, abs_dx, atol=1e-12)
    # wgrad: per_row_scale is indexed by ko, bias by the flattened (r, s, c)
    cols = g["R"] * g["S"] * g["C"]
    rs = rand_bits((g["Ko"],), "f32", 502).astype(np.float32)
    bc = rand_bits((cols,), "f32", 503).astype(np.float32)
    dw, s_w = oracle.conv2d_wgrad(dy, "bf16", x, "bf16", *geom_args(g), chain=[("per_row_scale", rs, "f32"), ("bias", bc, "f32")],
                                  want_abs=True, **geom_kw(g))
    plain = oracle.conv2d_wgrad(dy, "bf16", x, "bf16", *geom_args(g), **geom_kw(g))
    np.testing.assert_allclose(dw, plain * rs[:, None].astype(np.float64) + bc[None, :].astype(np.float64), atol=1e-12)
    sub = oracle.conv2d_wgrad(dy, "bf16", x, "bf16", *geom_args(g), rows=[1, 0], **geom_kw(g))
    assert np.array_equal(sub, plain[[1, 0]])
