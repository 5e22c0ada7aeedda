"""Run a synthetic workload dict (see the input generator's docstring) through the fp64 oracle.

TEST INFRASTRUCTURE: imported by tests, the smoke check and the benchmark's CPU-baseline leg only.
"""
import numpy as np

from . import batched_gemm, conv2d_dgrad, conv2d_fprop, conv2d_wgrad, gemm, grouped_gemm

_TENSOR_OPS = {"bias", "per_col_scale", "row_broadcast", "per_row_scale", "column_broadcast",
               "aux_load"}


def _chain(spec, row_offset=0, n_rows=None, group=None):
    """Resolve tensor names; matrices and m-indexed vectors are sliced to the rows a sub-problem
    (group) covers, and of a [groups, N padded] array of n-indexed vectors group g takes row g."""
    out = []
    for st in spec["epilogue"]:
        name = st[0]
        if name in _TENSOR_OPS:
            arr, dt = spec["tensors"][st[1]]
            if group is not None and name in ("bias", "per_col_scale", "row_broadcast"):
                arr = np.ascontiguousarray(arr[group, :spec["N"]])
            if name == "aux_load" and n_rows is not None:
                arr = np.ascontiguousarray(arr[row_offset:row_offset + n_rows])
            if name in ("per_row_scale", "column_broadcast") and n_rows is not None:
                arr = np.ascontiguousarray(arr[row_offset:row_offset + n_rows])
            out.append((name, arr, dt) + tuple(st[2:]))
        else:
            out.append(tuple(st))
    return out


def run(spec, rows=None, want_abs=False):
    """Unrounded float64 result.  gemm / conv: [M or len(rows), N]; batched: [batch, M, N];
    grouped: packed [sum M_g, N]."""
    op = spec["op"]
    if op == "gemm":
        return gemm(spec["A"], spec["dt_in"], spec["a_strides"], spec["B"], spec["dt_in"],
                    spec["b_strides"], spec["M"], spec["N"], spec["K"], chain=_chain(spec),
                    rows=rows, want_abs=want_abs)
    if op == "batched_gemm":
        if rows is not None:
            raise ValueError("row sampling is per gemm / conv only")
        aux_bs = spec["M"] * spec["N"]
        return batched_gemm(spec["A"], spec["dt_in"], spec["a_strides"], spec["B"], spec["dt_in"],
                            spec["b_strides"], spec["batch"], spec["M"], spec["N"], spec["K"],
                            chain=_chain(spec), aux_bs=aux_bs, want_abs=want_abs)
    if op == "grouped_gemm":
        M_g = spec["M_g"]
        offs = np.concatenate([[0], np.cumsum(M_g)]).astype(int)
        A_list = [np.ascontiguousarray(spec["A"][offs[g]:offs[g + 1]]) for g in range(len(M_g))]
        B_list = [np.ascontiguousarray(spec["B"][g]) for g in range(len(M_g))]
        chains = [_chain(spec, offs[g], M_g[g], group=g) for g in range(len(M_g))]
        return grouped_gemm(A_list, spec["dt_in"], spec["a_strides"], B_list, spec["dt_in"],
                            spec["b_strides"], M_g, spec["N"], spec["K"], chains=chains,
                            want_abs=want_abs)
    if op == "conv2d_fprop":
        return conv2d_fprop(spec["x"], spec["dt_in"], spec["w"], spec["dt_in"], spec["Nb"], spec["H"],
                            spec["W"], spec["C"], spec["Ko"], spec["R"], spec["S"], pad=spec["pad"],
                            stride=spec["stride"], dil=spec["dil"], chain=_chain(spec), rows=rows,
                            want_abs=want_abs)
    if op in ("conv2d_dgrad", "conv2d_wgrad"):
        fn, other = (conv2d_dgrad, spec["w"]) if op == "conv2d_dgrad" else (conv2d_wgrad, spec["x"])
        return fn(spec["dy"], spec["dt_in"], other, spec["dt_in"], spec["Nb"], spec["H"], spec["W"], spec["C"],
                  spec["Ko"], spec["R"], spec["S"], pad=spec["pad"], stride=spec["stride"], dil=spec["dil"],
                  chain=_chain(spec), rows=rows, want_abs=want_abs)
    raise ValueError(op)
