"""Pins for oracle/run_spec.py, the glue that turns a synthetic workload dict into oracle calls:
every branch (gemm with row sampling, batched with a per-batch residual, grouped with per-group
vectors / packed residual / packed per-row vectors, conv with bias + residual) against numpy /
torch fp64 expressions written out here.  CPU only."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import run_spec
from paper_2603_29010_amd import synth


def val(a, dt):
    return synth.bits_to_f64(a, dt)


def tens(spec, prefix):
    (key,) = [k for k in spec["tensors"] if k.startswith(prefix)]
    arr, dt = spec["tensors"][key]
    return val(arr, dt)


def test_gemm_spec_layouts_epilogue_and_row_sampling():
    for a_layout, b_layout in (("row", "col"), ("row", "row"), ("col", "col"), ("col", "row")):
        spec = synth.gemm_spec(7, 5, 16, dt_in="f16", dt_out="f32", a_layout=a_layout, b_layout=b_layout,
                               epilogue=("bias", ("aux_load", 0.5), "relu"))
        A = val(spec["A"], "f16")
        B = val(spec["B"], "f16")
        A = A if a_layout == "row" else A.T
        B = B.T if b_layout == "col" else B
        ref = np.maximum(A @ B + tens(spec, "bias")[None, :] + 0.5 * tens(spec, "aux_load"), 0.0)
        got = run_spec.run(spec)
        np.testing.assert_allclose(got, ref, atol=1e-12)
        rows = [6, 0, 3]
        got_r, absacc = run_spec.run(spec, rows=rows, want_abs=True)
        np.testing.assert_allclose(got_r, ref[rows], atol=1e-12)
        np.testing.assert_allclose(absacc, (np.abs(A) @ np.abs(B))[rows], atol=1e-12)


def test_batched_spec_residual_advances_per_batch():
    spec = synth.batched_spec(3, 4, 6, 8, dt_out="f32", epilogue=[("scale", 0.25), "aux_load", "column_broadcast"])
    A, B = val(spec["A"], "f16"), val(spec["B"], "f16")
    res = tens(spec, "aux_load").reshape(3, 4, 6)
    col = tens(spec, "column_broadcast")          # indexed by the row within a batch
    ref = 0.25 * np.einsum("bmk,bnk->bmn", A, B) + res + col[None, :, None]
    np.testing.assert_allclose(run_spec.run(spec), ref, atol=1e-12)
    # B stored [b, K, N]
    spec = synth.batched_spec(2, 4, 8, 8, dt_out="f32", epilogue=[], b_layout="row", a_layout="col")
    ref = np.einsum("bkm,bkn->bmn", val(spec["A"], "f16"), val(spec["B"], "f16"))
    np.testing.assert_allclose(run_spec.run(spec), ref, atol=1e-12)


def test_grouped_spec_per_group_tensors():
    M_g = [3, 0, 5, 1]
    N, K = 5, 8                                    # N % 8 != 0: bias rows are padded to 8
    for b_layout in ("col", "row"):
        if b_layout == "row":
            N = 8
        spec = synth.grouped_spec(M_g, N, K, dt_out="f32", b_layout=b_layout,
                                  epilogue=("per_row_scale", "bias", ("aux_load", -2.0), "per_col_scale"))
        A = val(spec["A"], "bf16")
        Bs = val(spec["B"], "bf16")
        rs, bias, res, cs = tens(spec, "per_row_scale"), tens(spec, "bias"), tens(spec, "aux_load"), tens(spec, "per_col_scale")
        assert bias.shape == (4, 8) and cs.shape == (4, 8) and res.shape == (9, N) and rs.shape == (9,)
        parts, o = [], 0
        for g, m in enumerate(M_g):
            Bg = Bs[g].T if b_layout == "col" else Bs[g]
            pre = A[o:o + m] @ Bg
            parts.append((pre * rs[o:o + m, None] + bias[g, None, :N] - 2.0 * res[o:o + m]) * cs[g, None, :N])
            o += m
        ref = np.concatenate(parts)
        got = run_spec.run(spec)
        assert got.shape == (9, N)
        np.testing.assert_allclose(got, ref, atol=1e-12)
        # group g's bias must be row g: a spec whose rows are swapped gives a different answer
        assert not np.allclose(bias[0, :N], bias[2, :N])


def test_conv_spec_bias_residual_and_row_sampling():
    spec = synth.conv_spec(2, 6, 5, 8, 4, 3, 3, pad=(1, 2), stride=(2, 1), dil=(1, 2), dt_out="f32",
                           epilogue=("bias", "aux_load", "relu"))
    x = torch.from_numpy(val(spec["x"], "bf16")).permute(0, 3, 1, 2)           # NCHW
    w = torch.from_numpy(val(spec["w"], "bf16")).permute(0, 3, 1, 2)           # K C R S
    y = F.conv2d(x, w, padding=(1, 2), stride=(2, 1), dilation=(1, 2)).permute(0, 2, 3, 1).numpy()
    assert y.shape == (2, spec["P"], spec["Q"], 4)
    ref = np.maximum(y.reshape(-1, 4) + tens(spec, "bias")[None, :] + tens(spec, "aux_load"), 0.0)
    got = run_spec.run(spec)
    np.testing.assert_allclose(got, ref, atol=1e-12)
    rows = [spec["M"] - 1, 0, 7]
    np.testing.assert_allclose(run_spec.run(spec, rows=rows), ref[rows], atol=1e-12)
