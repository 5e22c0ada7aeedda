"""Shared helpers of the GPU parity tests: run a workload on both sides and compare."""
import numpy as np

import oracle
from oracle import run_spec as orc_run

EPS_OUT = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24}


def chain_gain(spec):
    """Upper bound on how much the chain amplifies an error of the accumulator."""
    g = 1.0
    for st in spec["epilogue"]:
        if st[0] == "scale":
            g *= abs(st[1])
        elif st[0] == "leaky_relu":
            g *= max(1.0, abs(st[1]))
        elif st[0] == "elu":
            g *= max(1.0, abs(st[1]))
        elif st[0] in ("per_row_scale", "per_col_scale"):
            arr, dt = spec["tensors"][st[1]]
            from paper_2603_29010_amd import synth
            g *= float(np.abs(synth.bits_to_f64(arr, dt)).max())
        elif st[0] in ("gelu_tanh", "gelu_erf", "silu", "mish", "hardswish"):
            g *= 1.2
    return g


def compare(got, ref, absacc, spec, label="", mandated=True):
    """The two bars: the mandated |gpu-ref| <= 1e-2 (|ref|+1), and a sharp one that a kernel
    skipping work could not pass: output rounding + worst-case fp32 accumulation error
    K 2^-24 sum|a||b| carried through the chain + fp32 epilogue arithmetic."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{label}: non-finite or unwritten output elements: {np.count_nonzero(~np.isfinite(got))}"
    err = np.abs(got - ref)
    # (mandated=False: inputs built to cancel -- sums far below sum|a||b| -- where only the bound that
    # knows sum|a||b| is meaningful)
    loose = 1e-2 * (np.abs(ref) + 1.0)
    assert not mandated or np.all(err <= loose), f"{label}: max err {err.max():.3e} exceeds 1e-2(|ref|+1) at {np.unravel_index(np.argmax(err - loose), err.shape)}"
    K = spec["K"]
    # 8-bit inputs: the matrix instruction sums 32 products at a time after aligning them to the largest
    # one and dropping what lies below 2^-13 of it (measured: 1 + 2^-13 is kept, 1 + 2^-14 is not), i.e.
    # less than 32 * 2^-13 * max|a b| <= 2^-8 * (the group's sum |a||b|) per instruction
    acc_eps = K * 2.0 ** -24 + (2.0 ** -8 if spec["dt_in"] in ("e4m3", "e5m2") else 0.0)
    sharp = (EPS_OUT[spec["dt_out"]] * np.abs(ref) + chain_gain(spec) * acc_eps * absacc
             + 2e-6 * (np.abs(ref) + 1.0))
    bad = err > sharp
    assert not bad.any(), (f"{label}: {bad.sum()} elements exceed the sharp bound; worst err {err[bad].max():.3e} "
                           f"vs bound {sharp[bad][np.argmax(err[bad])]:.3e} at {np.argwhere(bad)[0]}")
    return float(err.max())


def oracle_result(spec, rows=None):
    return orc_run.run(spec, rows=rows, want_abs=True)


def gpu_result(spec, tune=None):
    from paper_2603_29010_amd.workload import DeviceWorkload
    w = DeviceWorkload(spec)
    w.run(tune=tune)
    return w.result(), w


def check(spec, tune=None, rows=None, label="", mandated=True):
    got, w = gpu_result(spec, tune)
    # every element of the output must have been written (the buffer starts as NaN patterns), also
    # where the oracle is only asked for a sample of the rows
    assert np.all(np.isfinite(got)), f"{label}: {np.count_nonzero(~np.isfinite(got))} output elements unwritten or non-finite"
    ref, absacc = oracle_result(spec, rows=rows)
    if rows is not None:
        got = got[np.asarray(rows)]
    got = got.reshape(ref.shape)
    return compare(got, ref, absacc, spec, label, mandated)


def check_exact(spec, tune=None, label=""):
    """Integer-valued inputs, results exactly representable: the GPU must equal the oracle bit for bit."""
    got, w = gpu_result(spec, tune)
    ref = orc_run.run(spec)
    got = got.reshape(ref.shape)
    ref_r = oracle.round_to(ref, spec["dt_out"]).reshape(ref.shape)
    assert np.array_equal(ref_r, ref), "test set-up: expected values are not exactly representable"
    mism = np.argwhere(got != ref)
    assert mism.size == 0, f"{label}: {len(mism)} mismatches, first at {mism[0]}: gpu {got[tuple(mism[0])]} ref {ref[tuple(mism[0])]}"
