"""Pins for the fp64 CPU oracle: everything here checks the oracle against something
other than itself -- closed forms, library routines (numpy / torch CPU, fp64),
pure-Python brute force on tiny shapes, and the numbers the paper prints for its
worked SOL example.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2603_29010_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bits(x, dt):
    return synth.to_bits(np.asarray(x, dtype=np.float64), dt)


def val(a, dt):
    return synth.bits_to_f64(a, dt)


# ------------------------------------------------------------------ storage formats / rounding

def test_fp16_decode_matches_numpy_exhaustive():
    allbits = np.arange(65536, dtype=np.uint16)
    got = oracle.load(allbits, "f16")
    ref = allbits.view(np.float16).astype(np.float64)
    assert np.array_equal(got, ref, equal_nan=True)


def test_fp16_round_trip_exhaustive():
    allbits = np.arange(65536, dtype=np.uint16)
    v = allbits.view(np.float16).astype(np.float64)
    for b, x in zip(allbits.tolist(), v.tolist()):
        if math.isnan(x):
            continue
        assert oracle.encode16(x, "f16") == b


def test_bf16_encode_matches_torch_exhaustive():
    allbits = np.arange(65536, dtype=np.uint16)
    v = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    for b, x in zip(allbits.tolist(), v.tolist()):
        if math.isnan(x):
            continue
        assert oracle.encode16(x, "bf16") == b
    # and values between two bf16 numbers land on the nearest (ties to even), as torch casts them
    x = np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8, -3.1415926, 1e-40, 3.0e38, 65504.0])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert [oracle.encode16(float(np.float32(t)), "bf16") for t in x] == ref.tolist()


def test_bf16_decode_matches_torch_exhaustive():
    allbits = np.arange(65536, dtype=np.uint16)
    got = oracle.load(allbits, "bf16")
    ref = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref, equal_nan=True)


def _fp8_hand_table(ebits, mbits, bias, ieee_specials):
    """Value of every code of an 8-bit format from its definition, written out independently:
    (-1)^s 2^(e-bias) (1 + m/2^mbits), subnormals 2^(1-bias) m/2^mbits; IEEE-style formats keep the
    top exponent for inf / NaN, the other kind only gives up the all-ones code for NaN."""
    out = []
    for code in range(256):
        sgn = -1.0 if code & 0x80 else 1.0
        e = (code >> mbits) & ((1 << ebits) - 1)
        m = code & ((1 << mbits) - 1)
        top = (1 << ebits) - 1
        if ieee_specials and e == top:
            v = math.inf if m == 0 else math.nan
        elif not ieee_specials and e == top and m == (1 << mbits) - 1:
            v = math.nan
        elif e == 0:
            v = 2.0 ** (1 - bias) * (m / 2.0 ** mbits)
        else:
            v = 2.0 ** (e - bias) * (1 + m / 2.0 ** mbits)
        out.append(sgn * v)
    return np.array(out)


def test_fp8_decode_every_code_against_hand_table_and_torch():
    codes = np.arange(256, dtype=np.uint8)
    for name, tdt, table in (("e4m3", torch.float8_e4m3fn, _fp8_hand_table(4, 3, 7, False)),
                             ("e5m2", torch.float8_e5m2, _fp8_hand_table(5, 2, 15, True))):
        got = oracle.load(codes, name)
        assert np.array_equal(got, table, equal_nan=True), name
        ref = torch.from_numpy(codes).view(tdt).to(torch.float64).numpy()
        assert np.array_equal(got, ref, equal_nan=True), name
    e4 = oracle.load(codes, "e4m3")
    assert np.nanmax(e4) == 448.0 and e4[0x08] == 2.0 ** -6 and e4[0x01] == 2.0 ** -9 and e4[0x38] == 1.0
    e5 = oracle.load(codes, "e5m2")
    assert e5[0x7B] == 57344.0 and e5[0x7C] == math.inf and e5[0x3C] == 1.0 and e5[0x01] == 2.0 ** -16


def test_gemm_with_fp8_inputs_matches_numpy():
    rng = np.random.default_rng(5)
    for dt in ("e4m3", "e5m2"):
        A = synth.to_bits(rng.standard_normal((5, 16)), dt)
        B = synth.to_bits(rng.standard_normal((4, 16)), dt)
        assert A.dtype == np.uint8
        D = oracle.gemm(A, dt, (16, 1), B, dt, (1, 16), 5, 4, 16)
        np.testing.assert_allclose(D, val(A, dt) @ val(B, dt).T, atol=1e-12)


def test_batched_gemm_with_fp8_inputs_advances_by_one_byte_elements():
    rng = np.random.default_rng(6)
    A = synth.to_bits(rng.standard_normal((3, 5, 16)), "e5m2")
    B = synth.to_bits(rng.standard_normal((3, 4, 16)), "e5m2")
    D = oracle.batched_gemm(A, "e5m2", (16, 1, 80), B, "e5m2", (1, 16, 64), 3, 5, 4, 16)
    np.testing.assert_allclose(D, np.einsum("bmk,bnk->bmn", val(A, "e5m2"), val(B, "e5m2")), atol=1e-12)


def test_grouped_gemm_with_fp8_inputs_matches_numpy_per_group():
    rng = np.random.default_rng(8)
    M_g, N, K = [4, 0, 7], 5, 32
    for dt in ("e4m3", "e5m2"):
        A = [synth.to_bits(rng.standard_normal((m, K)), dt) for m in M_g]
        B = [synth.to_bits(rng.standard_normal((N, K)), dt) for _ in M_g]
        D = oracle.grouped_gemm(A, dt, (K, 1), B, dt, (1, K), M_g, N, K)
        ref = np.concatenate([val(a, dt) @ val(b, dt).T for a, b in zip(A, B)])
        np.testing.assert_allclose(D, ref, atol=1e-12)


def test_rounding_ties_and_double_rounding():
    r = oracle.round_to
    # bf16 has 8 significant bits: spacing 2^-7 in [1,2)
    assert r([1 + 2 ** -8], "bf16")[0] == 1.0                      # tie -> even (mantissa 0)
    assert r([1 + 3 * 2 ** -8], "bf16")[0] == 1 + 2 ** -6          # tie -> even (mantissa 2)
    assert r([1 + 2 ** -8 + 2 ** -40], "bf16")[0] == 1 + 2 ** -7   # just above the tie: must go up
    #   (rounding first to fp32 would land on the tie and then wrongly go down)
    assert r([-(1 + 2 ** -8 + 2 ** -40)], "bf16")[0] == -(1 + 2 ** -7)
    # fp16: 11 significant bits, max finite 65504, overflow threshold 65520
    assert r([65519.99], "f16")[0] == 65504.0
    assert np.isinf(r([65520.0], "f16")[0])
    assert r([2 ** -25], "f16")[0] == 0.0                           # half the smallest subnormal: tie -> 0
    assert r([2 ** -25 * 1.001], "f16")[0] == 2 ** -24
    assert r([1 + 2 ** -11], "f16")[0] == 1.0
    assert r([1 + 3 * 2 ** -11], "f16")[0] == 1 + 2 ** -9
    # fp32
    assert r([1 + 2 ** -24], "f32")[0] == 1.0
    assert r([1 + 2 ** -24 + 2 ** -50], "f32")[0] == 1 + 2 ** -23


def test_rounding_matches_library_casts():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-8, 8, 20000),
                        [0.0, -0.0, 1e-45, 3e38, 7e4, 6e-8]])
    assert np.array_equal(oracle.round_to(x, "f32"), x.astype(np.float32).astype(np.float64))
    x16 = x[np.abs(x) < 6e4]
    assert np.array_equal(oracle.round_to(x16, "f16"), x16.astype(np.float16).astype(np.float64))
    # torch's float32 -> bfloat16 cast is round-to-nearest-even; feed it exact float32 values
    xf = x.astype(np.float32)
    ref = torch.from_numpy(xf).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_to(xf.astype(np.float64), "bf16"), ref)


# ------------------------------------------------------------------ epilogue ops

ACT_CASES = np.array([-30.0, -6.0, -3.0, -2.5, -1.0, -0.3, 0.0, 0.2, 1.0, 2.9, 3.0, 7.0, 30.0])


def _torch_ref(name, x):
    t = torch.tensor(x, dtype=torch.float64)
    return {
        "relu": lambda: F.relu(t),
        "gelu_tanh": lambda: F.gelu(t, approximate="tanh"),
        "gelu_erf": lambda: F.gelu(t),
        "silu": lambda: F.silu(t),
        "sigmoid": lambda: torch.sigmoid(t),
        "tanh": lambda: torch.tanh(t),
        "mish": lambda: F.mish(t),
        "hardswish": lambda: F.hardswish(t),
    }[name]().numpy()


@pytest.mark.parametrize("name", ["relu", "gelu_tanh", "gelu_erf", "silu", "sigmoid", "tanh", "mish",
                                  "hardswish"])
def test_activation_matches_torch_fp64(name):
    got = np.array([oracle.epilogue(v, 0, 0, [(name,)]) for v in ACT_CASES])
    np.testing.assert_allclose(got, _torch_ref(name, ACT_CASES), rtol=1e-13, atol=1e-300)


def test_activation_golden_values():
    # fp64 textbook values, file tests/golden/activations.txt (computed with mpmath-free closed forms)
    for line in open(os.path.join(GOLD, "activations.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        name, x, y = line.split()
        assert oracle.epilogue(float(x), 0, 0, [(name,)]) == pytest.approx(float(y), rel=1e-14, abs=1e-300)


def test_parametric_activations():
    e = oracle.epilogue
    t = torch.tensor(ACT_CASES, dtype=torch.float64)
    got = np.array([e(v, 0, 0, [("leaky_relu", 0.1)]) for v in ACT_CASES])
    np.testing.assert_allclose(got, F.leaky_relu(t, 0.1).numpy(), rtol=1e-15)
    got = np.array([e(v, 0, 0, [("elu", 1.5)]) for v in ACT_CASES])
    np.testing.assert_allclose(got, F.elu(t, 1.5).numpy(), rtol=1e-14)
    got = np.array([e(v, 0, 0, [("clamp", -0.5, 6.0)]) for v in ACT_CASES])
    np.testing.assert_array_equal(got, np.clip(ACT_CASES, -0.5, 6.0))
    assert e(3.0, 0, 0, [("scale", -0.25)]) == -0.75


def test_chain_is_applied_left_to_right_with_coordinates():
    bias = bits([10.0, 20.0, 30.0], "f32")           # indexed by n
    rowv = bits([2.0, 4.0], "f32")                   # indexed by m
    aux = bits([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]], "f32")
    e = oracle.epilogue
    # order matters: relu(v + b) vs relu(v) + b
    assert e(-15.0, 0, 0, [("bias", bias, "f32"), ("relu",)]) == 0.0
    assert e(-15.0, 0, 0, [("relu",), ("bias", bias, "f32")]) == 10.0
    # coordinates: bias / per_col / row_broadcast use n; per_row / column_broadcast use m
    assert e(1.0, 1, 2, [("bias", bias, "f32")]) == 31.0
    assert e(1.0, 1, 2, [("row_broadcast", bias, "f32")]) == 31.0
    assert e(1.0, 1, 2, [("per_col_scale", bias, "f32")]) == 30.0
    assert e(1.0, 1, 2, [("per_row_scale", rowv, "f32")]) == 4.0
    assert e(1.0, 1, 2, [("column_broadcast", rowv, "f32")]) == 5.0
    assert e(1.0, 1, 2, [("aux_load", aux, "f32")]) == 7.0          # aux[1,2] = 6
    assert e(1.0, 1, 0, [("aux_load", aux, "f32", 0.5)]) == 3.0     # 1 + 0.5*4
    # alpha/beta scaling of the paper's `.with_scaling`: alpha*acc + beta*C
    assert e(2.0, 0, 1, [("scale", 3.0), ("aux_load", aux, "f32", -2.0)]) == 2.0
    # aux_store captures the value at its position in the chain, rounded to the aux format
    store = np.zeros((2, 3))
    out = e(1 + 2 ** -8 + 2 ** -40, 1, 1, [("scale", 1.0), ("aux_store", store, "bf16"), ("scale", 2.0)])
    assert store[1, 1] == 1 + 2 ** -7 and out == 2 * (1 + 2 ** -8 + 2 ** -40)
    assert np.count_nonzero(store) == 1


# ------------------------------------------------------------------ GEMM

def _rand_bits(shape, dt, seed):
    rng = np.random.default_rng(seed)
    return bits(rng.standard_normal(shape), dt)


def test_gemm_closed_forms():
    K = 37
    A = bits(np.ones((5, K)), "bf16")
    B = bits(np.ones((K, 7)), "bf16")
    D = oracle.gemm(A, "bf16", (K, 1), B, "bf16", (7, 1), 5, 7, K)
    assert np.array_equal(D, np.full((5, 7), float(K)))
    # identity
    n = 9
    Bm = _rand_bits((n, n), "f16", 1)
    D = oracle.gemm(bits(np.eye(n), "f16"), "f16", (n, 1), Bm, "f16", (n, 1), n, n, n)
    assert np.array_equal(D, val(Bm, "f16"))
    # K = 1: outer product
    a = _rand_bits((6, 1), "f32", 2)
    b = _rand_bits((1, 4), "f32", 3)
    D = oracle.gemm(a, "f32", (1, 1), b, "f32", (4, 1), 6, 4, 1)
    assert np.array_equal(D, val(a, "f32") * val(b, "f32"))


def test_gemm_brute_force_python_tiny():
    for (M, N, K) in [(1, 1, 1), (2, 3, 4), (3, 2, 5), (5, 4, 3)]:
        Ai = np.arange(M * K).reshape(M, K) % 5 - 2
        Bi = (np.arange(K * N).reshape(K, N) * 3) % 7 - 3
        want = [[sum(int(Ai[m, k]) * int(Bi[k, n]) for k in range(K)) for n in range(N)] for m in range(M)]
        D = oracle.gemm(bits(Ai, "bf16"), "bf16", (K, 1), bits(Bi, "bf16"), "bf16", (N, 1), M, N, K)
        assert D.tolist() == [[float(v) for v in row] for row in want]


@pytest.mark.parametrize("a_layout,b_layout", list(itertools.product(["row", "col"], ["row", "col"])))
@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_gemm_matches_numpy_all_layouts(a_layout, b_layout, dt):
    M, N, K = 13, 11, 17
    Am = _rand_bits((M, K), dt, 10)
    Bm = _rand_bits((K, N), dt, 11)
    ref = val(Am, dt) @ val(Bm, dt)
    A_st = np.ascontiguousarray(Am if a_layout == "row" else Am.T)
    B_st = np.ascontiguousarray(Bm if b_layout == "row" else Bm.T)
    a_str = (K, 1) if a_layout == "row" else (1, M)
    b_str = (N, 1) if b_layout == "row" else (1, K)
    D, S = oracle.gemm(A_st, dt, a_str, B_st, dt, b_str, M, N, K, want_abs=True)
    np.testing.assert_allclose(D, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(S, np.abs(val(Am, dt)) @ np.abs(val(Bm, dt)), rtol=1e-13)


def test_gemm_transpose_identity():
    # (A.B)^T = B^T.A^T: swapping the operands' roles and strides must give the transposed result
    M, N, K = 7, 5, 9
    A = _rand_bits((M, K), "bf16", 20)
    B = _rand_bits((K, N), "bf16", 21)
    D = oracle.gemm(A, "bf16", (K, 1), B, "bf16", (N, 1), M, N, K)
    Dt = oracle.gemm(B, "bf16", (1, N), A, "bf16", (1, K), N, M, K)
    assert np.array_equal(Dt, D.T)


def test_gemm_row_subset_and_epilogue_coordinates():
    M, N, K = 12, 6, 8
    A = _rand_bits((M, K), "bf16", 30)
    B = _rand_bits((N, K), "bf16", 31)
    bias = _rand_bits((N,), "bf16", 32)
    res = _rand_bits((M, N), "bf16", 33)
    chain = [("bias", bias, "bf16"), ("aux_load", res, "bf16"), ("relu",)]
    full = oracle.gemm(A, "bf16", (K, 1), B, "bf16", (1, K), M, N, K, chain=chain)
    ref = np.maximum(val(A, "bf16") @ val(B, "bf16").T + val(bias, "bf16")[None, :] + val(res, "bf16"), 0)
    np.testing.assert_allclose(full, ref, atol=1e-12)
    rows = [11, 0, 5]
    sub = oracle.gemm(A, "bf16", (K, 1), B, "bf16", (1, K), M, N, K, chain=chain, rows=rows)
    assert np.array_equal(sub, full[rows])


# ------------------------------------------------------------------ batched / grouped

def test_batched_matches_numpy_and_batch_strides():
    b, M, N, K = 3, 5, 4, 6
    A = _rand_bits((b, M, K), "f16", 40)
    B = _rand_bits((b, N, K), "f16", 41)
    D = oracle.batched_gemm(A, "f16", (K, 1, M * K), B, "f16", (1, K, N * K), b, M, N, K,
                            chain=[("scale", 0.5)])
    ref = 0.5 * np.einsum("bmk,bnk->bmn", val(A, "f16"), val(B, "f16"))
    np.testing.assert_allclose(D, ref, atol=1e-12)
    # batch stride 0 on B = one shared B
    D0 = oracle.batched_gemm(A, "f16", (K, 1, M * K), B, "f16", (1, K, 0), b, M, N, K)
    ref0 = np.einsum("bmk,nk->bmn", val(A, "f16"), val(B, "f16")[0])
    np.testing.assert_allclose(D0, ref0, atol=1e-12)
    # batch = 1 is a plain gemm
    D1 = oracle.batched_gemm(A[:1], "f16", (K, 1, M * K), B[:1], "f16", (1, K, N * K), 1, M, N, K)
    G1 = oracle.gemm(A[0], "f16", (K, 1), B[0], "f16", (1, K), M, N, K)
    assert np.array_equal(D1[0], G1)


def test_batched_aux_advances_per_batch():
    b, M, N, K = 2, 3, 4, 5
    A = _rand_bits((b, M, K), "f16", 42)
    B = _rand_bits((b, N, K), "f16", 43)
    R = _rand_bits((b * M, N), "f32", 44)
    D = oracle.batched_gemm(A, "f16", (K, 1, M * K), B, "f16", (1, K, N * K), b, M, N, K,
                            chain=[("aux_load", R, "f32")], aux_bs=M * N)
    ref = np.einsum("bmk,bnk->bmn", val(A, "f16"), val(B, "f16")) + val(R, "f32").reshape(b, M, N)
    np.testing.assert_allclose(D, ref, atol=1e-12)


def test_grouped_matches_numpy_per_group():
    M_g = [3, 0, 5, 1]
    N, K = 4, 6
    A = [_rand_bits((m, K), "bf16", 50 + i) for i, m in enumerate(M_g)]
    B = [_rand_bits((N, K), "bf16", 60 + i) for i in range(len(M_g))]
    D = oracle.grouped_gemm(A, "bf16", (K, 1), B, "bf16", (1, K), M_g, N, K,
                            chains=[[("silu",)]] * len(M_g))
    pre = np.concatenate([val(a, "bf16") @ val(b, "bf16").T for a, b in zip(A, B)])
    ref = pre / (1 + np.exp(-pre))
    assert D.shape == (sum(M_g), N)
    np.testing.assert_allclose(D, ref, atol=1e-12)
    # equal sizes == batched
    A2 = [_rand_bits((3, K), "bf16", 70 + i) for i in range(3)]
    D2 = oracle.grouped_gemm(A2, "bf16", (K, 1), B[:3], "bf16", (1, K), [3, 3, 3], N, K)
    Bt = oracle.batched_gemm(np.stack(A2), "bf16", (K, 1, 3 * K), np.stack(B[:3]), "bf16", (1, K, N * K),
                             3, 3, N, K)
    assert np.array_equal(D2, Bt.reshape(9, N))


# ------------------------------------------------------------------ conv2d fprop

def _conv(x, w, **kw):
    Nb, H, W, C = x.shape
    Ko, R, S, _ = w.shape
    return oracle.conv2d_fprop(x, "bf16", w, "bf16", Nb, H, W, C, Ko, R, S, **kw)


def test_conv_all_ones_counts_taps():
    C = 3
    x = bits(np.ones((1, 5, 6, C)), "bf16")
    w = bits(np.ones((2, 3, 3, C)), "bf16")
    y = _conv(x, w, pad=(1, 1)).reshape(1, 5, 6, 2)
    assert np.all(y[0, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[0, 0, 1:-1] == 6 * C) and np.all(y[0, 1:-1, 0] == 6 * C)
    assert np.all(y[0, -1, 1:-1] == 6 * C) and np.all(y[0, 1:-1, -1] == 6 * C)
    for h, ww in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[0, h, ww] == 4 * C)


def test_conv_delta_and_one_hot_taps_fix_orientation():
    C = 4
    x = _rand_bits((2, 5, 5, C), "bf16", 80)
    xv = val(x, "bf16")
    w = np.zeros((C, 3, 3, C))
    for c in range(C):
        w[c, 1, 1, c] = 1.0
    y = _conv(x, bits(w, "bf16"), pad=(1, 1)).reshape(2, 5, 5, C)
    assert np.array_equal(y, xv)                                   # centre tap: copy
    # tap (r=0, s=2): y[p,q] = x[p-1, q+1]  (cross-correlation: the filter is NOT flipped)
    w = np.zeros((C, 3, 3, C))
    for c in range(C):
        w[c, 0, 2, c] = 1.0
    y = _conv(x, bits(w, "bf16"), pad=(1, 1)).reshape(2, 5, 5, C)
    want = np.zeros_like(xv)
    want[:, 1:, :-1] = xv[:, :-1, 1:]
    assert np.array_equal(y, want)


def test_conv_1x1_is_gemm():
    Nb, H, W, C, Ko = 2, 3, 4, 8, 5
    x = _rand_bits((Nb, H, W, C), "bf16", 81)
    w = _rand_bits((Ko, 1, 1, C), "bf16", 82)
    y = _conv(x, w, pad=(0, 0))
    g = val(x, "bf16").reshape(-1, C) @ val(w, "bf16").reshape(Ko, C).T
    np.testing.assert_allclose(y, g, atol=1e-12)


def test_conv_h1_is_1d_correlation():
    W, S = 11, 4
    x = _rand_bits((1, 1, W, 1), "bf16", 83)
    w = _rand_bits((1, 1, S, 1), "bf16", 84)
    y = _conv(x, w, pad=(0, 0)).reshape(-1)
    ref = np.correlate(val(x, "bf16").reshape(-1), val(w, "bf16").reshape(-1), mode="valid")
    np.testing.assert_allclose(y, ref, atol=1e-13)


@pytest.mark.parametrize("pad,stride,dil,R,S", [((1, 1), (1, 1), (1, 1), 3, 3), ((0, 2), (2, 1), (1, 1), 3, 2),
                                                  ((2, 1), (1, 2), (2, 1), 3, 3), ((3, 3), (3, 2), (1, 2), 5, 4)])
def test_conv_matches_torch_fp64(pad, stride, dil, R, S):
    Nb, H, W, C, Ko = 2, 9, 8, 5, 4
    x = _rand_bits((Nb, H, W, C), "bf16", 85)
    w = _rand_bits((Ko, R, S, C), "bf16", 86)
    bias = _rand_bits((Ko,), "bf16", 87)
    y = _conv(x, w, pad=pad, stride=stride, dil=dil, chain=[("bias", bias, "bf16")])
    xt = torch.from_numpy(val(x, "bf16")).permute(0, 3, 1, 2)
    wt = torch.from_numpy(val(w, "bf16")).permute(0, 3, 1, 2)
    ref = F.conv2d(xt, wt, torch.from_numpy(val(bias, "bf16")), stride=stride, padding=pad, dilation=dil)
    P, Q = ref.shape[2], ref.shape[3]
    assert P == oracle.conv_out_dim(H, pad[0], dil[0], R, stride[0])
    assert Q == oracle.conv_out_dim(W, pad[1], dil[1], S, stride[1])
    np.testing.assert_allclose(y.reshape(Nb, P, Q, Ko), ref.permute(0, 2, 3, 1).numpy(), atol=1e-12)
    rows = [Nb * P * Q - 1, 0, 7]
    ysub = _conv(x, w, pad=pad, stride=stride, dil=dil, chain=[("bias", bias, "bf16")], rows=rows)
    assert np.array_equal(ysub, y[rows])


def test_conv_equals_explicit_im2col_times_matrix():
    Nb, H, W, C, Ko, R, S = 1, 4, 5, 2, 3, 3, 3
    x = _rand_bits((Nb, H, W, C), "bf16", 88)
    w = _rand_bits((Ko, R, S, C), "bf16", 89)
    xv = val(x, "bf16")
    cols = np.zeros((Nb * H * W, R * S * C))
    for n, p, q, r, s in itertools.product(range(Nb), range(H), range(W), range(R), range(S)):
        h, ww = p - 1 + r, q - 1 + s
        if 0 <= h < H and 0 <= ww < W:
            cols[(n * H + p) * W + q, (r * S + s) * C:(r * S + s + 1) * C] = xv[n, h, ww]
    ref = cols @ val(w, "bf16").reshape(Ko, -1).T
    np.testing.assert_allclose(_conv(x, w, pad=(1, 1)), ref, atol=1e-12)


# ------------------------------------------------------------------ SOL analysis: the paper's worked example

def _gold(path):
    d = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = [t.strip() for t in line.split("=")]
            d[k] = v
    return d


# ---- transform stage: transpose(tensor, NCL, NLC [, dtype_in, dtype_out]) ------------------------

@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_transpose_matches_numpy_and_index_loop(dt):
    batch, rows, cols = 3, 5, 7
    x = bits(synth.normal(11, 1, batch * rows * cols), dt).reshape(batch, rows, cols)
    got = oracle.transpose(x, dt, batch, rows, cols)
    assert got.shape == (batch, cols, rows)
    # numpy's own transposition of the decoded values
    assert np.array_equal(got, np.swapaxes(val(x, dt), 1, 2))
    # the definition, index by index
    v = val(x, dt)
    for b, r, c in itertools.product(range(batch), range(rows), range(cols)):
        assert got[b, c, r] == v[b, r, c]


def test_transpose_twice_is_identity_and_vectors_are_copies():
    batch, rows, cols = 2, 6, 4
    x = synth.normal(12, 1, batch * rows * cols).astype(np.float32).reshape(batch, rows, cols)
    once = oracle.transpose(x, "f32", batch, rows, cols)
    twice = oracle.transpose(once.astype(np.float32), "f32", batch, cols, rows)
    assert np.array_equal(twice, x.astype(np.float64))
    # a single row or a single column: the element order in memory does not change
    row = synth.normal(13, 1, 9).astype(np.float32)
    assert np.array_equal(oracle.transpose(row.reshape(1, 1, 9), "f32", 1, 1, 9).reshape(-1), row)
    assert np.array_equal(oracle.transpose(row.reshape(1, 9, 1), "f32", 1, 9, 1).reshape(-1), row)
    # NCHW -> NHWC of a tensor whose value encodes its index (n, c, h, w)
    N, Cc, H, W = 2, 3, 2, 2
    idx = np.arange(N * Cc * H * W, dtype=np.float32).reshape(N, Cc, H * W)
    nhwc = oracle.transpose(idx, "f32", N, Cc, H * W).reshape(N, H, W, Cc)
    for n, c, h, w in itertools.product(range(N), range(Cc), range(H), range(W)):
        assert nhwc[n, h, w, c] == ((n * Cc + c) * H + h) * W + w
    assert oracle.transpose(np.empty((0, 4, 4), np.float32), "f32", 0, 4, 4).size == 0


def test_transpose_with_conversion_rounds_once_to_nearest_even():
    # fp32 -> bf16 / fp16: the unrounded transposition followed by round_to equals the library casts
    x = (synth.normal(14, 1, 4 * 8) * 3.0).astype(np.float32).reshape(1, 4, 8)
    t = oracle.transpose(x, "f32", 1, 4, 8)
    want16 = torch.from_numpy(x).transpose(1, 2).contiguous()
    assert np.array_equal(oracle.round_to(t, "f16"), want16.to(torch.float16).to(torch.float64).numpy())
    assert np.array_equal(oracle.round_to(t, "bf16"), want16.to(torch.bfloat16).to(torch.float64).numpy())
    # a tie: 1 + 2^-8 is halfway between two bf16 values and goes to the even one (1.0)
    tie = np.array([[[1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]]], dtype=np.float32)
    assert list(oracle.round_to(oracle.transpose(tie, "f32", 1, 1, 2), "bf16").reshape(-1)) == [1.0, 1.0 + 2.0 ** -6]


def test_sol_reproduces_paper_worked_example():
    g = _gold(os.path.join(GOLD, "sol_report_example.txt"))
    n = int(g["n"])
    flops = oracle.gemm_flops(1, n, n, n)
    nbytes = 3 * n * n * int(g["bytes_per_element"])
    assert flops == int(g["total_flops"])
    assert nbytes == int(g["total_bytes"])
    ratio = float(g["sm_clock_mhz"]) / float(g["max_sm_clock_mhz"])
    assert round(ratio, 4) == float(g["clock_ratio"])
    s = oracle.sol_bound(flops, nbytes, float(g["tf32_peak_tflops_at_max"]) * 1e12, ratio,
                         float(g["hbm_tbps"]) * 1e12, 1.0)
    # the paper divides the figures it rounded for print (1.374e11 / 2.013e8 = 682.56 -> "682.6");
    # the exact ratio is 2N/12 * ... = 682.67, so allow 0.1
    assert s["ai"] == pytest.approx(float(g["ai"]), abs=0.1)
    assert s["ai"] == pytest.approx(2 * n / 12.0)
    # the paper rounds the clock ratio to 0.7576 before scaling; allow its last printed digit
    assert s["peak_flops"] / 1e12 == pytest.approx(float(g["tf32_peak_tflops_effective"]), abs=0.02)
    assert round(s["t_compute"] * 1e3, 3) == float(g["t_compute_ms"])
    assert round(s["t_mem"] * 1e3, 3) == float(g["t_mem_ms"])
    assert round(s["t_sol"] * 1e3, 3) == float(g["t_sol_ms"])
    assert round(s["t_compute"] * 1e3, 4) == float(g["t_compute_ms_tf32_4dp"])
    assert round(s["t_mem"] * 1e3, 4) == float(g["t_mem_ms_4dp"])
    assert s["ridge"] == pytest.approx(float(g["ridge"]), abs=0.06)
    assert s["compute_bound"] == 1 and g["bottleneck"] == "compute"
    s16 = oracle.sol_bound(flops, nbytes, float(g["fp16_peak_tflops_at_max"]) * 1e12, ratio,
                           float(g["hbm_tbps"]) * 1e12, 1.0)
    assert s16["peak_flops"] / 1e12 == pytest.approx(float(g["fp16_peak_tflops_effective"]), abs=0.03)
    assert round(s16["t_sol"] * 1e3, 4) == float(g["t_sol_ms_fp16"])
    assert s16["t_mem"] == s["t_mem"]                 # traffic unchanged in the FP16 variant


def test_sol_memory_bound_side():
    s = oracle.sol_bound(1e9, 1e9, 1e15, 1.0, 1e12, 0.5)
    assert s["t_sol"] == s["t_mem"] == 1e9 / 0.5e12 and s["compute_bound"] == 0
