"""fp64 CPU oracle -- TEST INFRASTRUCTURE, not product code.

ctypes front end of ``ucl_oracle.c`` (plain C, fp64).  Only ``tests/``, the
smoke check and the benchmark's CPU-baseline leg may import this package; the
GPU library never does, and this package never imports the GPU library.

Arrays go in as numpy arrays holding the *stored bit patterns*:
``uint8`` for the 8-bit formats (``"e4m3"``, ``"e5m2"``), ``uint16`` for bf16 / fp16
(with ``dtype="bf16"`` or ``"f16"``), ``float32`` or
``float64`` otherwise.  Results come back as unrounded ``float64``; use
``round_to`` for the value the output format would store.

An epilogue chain is a list of steps, each a tuple ``(name, *args)``:
  ("scale", alpha) ("bias", vec, dtype) ("aux_load", mat, dtype[, beta])
  ("relu",) ("gelu_tanh",) ("gelu_erf",) ("silu",) ("sigmoid",) ("tanh",)
  ("mish",) ("hardswish",) ("leaky_relu", alpha) ("elu", alpha)
  ("clamp", lo, hi) ("per_row_scale", vec, dtype) ("per_col_scale", vec, dtype)
  ("row_broadcast", vec, dtype) ("column_broadcast", vec, dtype)
  ("aux_store", out_float64_matrix, dtype)
following the paper's grammar rule ``epilogue_op``.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ucl_oracle.c")
_LIB = os.path.join(_HERE, "libucl_oracle.so")

DT = {"e4m3": 8, "e5m2": 9, "bf16": 16, "f16": 17, "f32": 32, "f64": 64}
_OPS = {
    "scale": 1, "bias": 2, "aux_load": 3, "relu": 4, "gelu_tanh": 5, "gelu_erf": 6,
    "silu": 7, "sigmoid": 8, "tanh": 9, "mish": 10, "hardswish": 11, "leaky_relu": 12,
    "elu": 13, "clamp": 14, "per_row_scale": 15, "per_col_scale": 16,
    "row_broadcast": 17, "column_broadcast": 18, "aux_store": 19,
}
_VEC_OPS = {"bias", "per_row_scale", "per_col_scale", "row_broadcast", "column_broadcast"}


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP over output rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-D_GNU_SOURCE",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Step(C.Structure):
    _fields_ = [("op", C.c_int32), ("dtype", C.c_int32), ("p0", C.c_double), ("p1", C.c_double),
                ("ptr", C.c_void_p), ("ld", C.c_int64)]


class _Chain(C.Structure):
    _fields_ = [("n_steps", C.c_int32), ("pad_", C.c_int32), ("steps", _Step * 16)]


class _Sol(C.Structure):
    _fields_ = [("flops", C.c_double), ("bytes", C.c_double), ("peak_flops", C.c_double),
                ("peak_bw", C.c_double), ("ai", C.c_double), ("ridge", C.c_double),
                ("t_compute", C.c_double), ("t_mem", C.c_double), ("t_sol", C.c_double),
                ("compute_bound", C.c_int32), ("pad_", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_round.restype = C.c_double
        _lib.orc_round.argtypes = [C.c_double, C.c_int]
        _lib.orc_load.restype = C.c_double
        _lib.orc_load.argtypes = [C.c_void_p, C.c_int, C.c_int64]
        _lib.orc_encode16.restype = C.c_uint16
        _lib.orc_encode16.argtypes = [C.c_double, C.c_int]
        _lib.orc_epilogue.restype = C.c_double
        _lib.orc_epilogue.argtypes = [C.c_double, C.c_int64, C.c_int64, C.c_void_p]
        _lib.orc_conv_out_dim.restype = C.c_int64
        _lib.orc_conv_out_dim.argtypes = [C.c_int64] * 5
        _lib.orc_gemm_flops.restype = C.c_double
        _lib.orc_gemm_flops.argtypes = [C.c_double] * 4
        _lib.orc_transpose.restype = None
        _lib.orc_transpose.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p]
        _lib.orc_sol_bound.restype = None
        _lib.orc_sol_bound.argtypes = [C.c_double] * 6 + [C.c_void_p]
    return _lib


def _ptr(a):
    return C.c_void_p(a.ctypes.data)


def _check(a, dtype):
    want = {"e4m3": np.uint8, "e5m2": np.uint8, "bf16": np.uint16, "f16": np.uint16, "f32": np.float32,
            "f64": np.float64}[dtype]
    if a.dtype != want:
        raise TypeError(f"array for {dtype} must be {want}, got {a.dtype}")
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("oracle arrays must be C-contiguous (pass strides explicitly)")
    return a


def _chain(steps, keep):
    """Translate a python chain into the C struct; `keep` holds array refs alive."""
    if not steps:
        return None
    c = _Chain()
    c.n_steps = len(steps)
    for i, st in enumerate(steps):
        name = st[0]
        s = c.steps[i]
        s.op = _OPS[name]
        if name in ("scale", "leaky_relu", "elu"):
            s.p0 = float(st[1])
        elif name == "clamp":
            s.p0, s.p1 = float(st[1]), float(st[2])
        elif name in _VEC_OPS:
            arr = _check(st[1], st[2]); keep.append(arr)
            s.ptr = arr.ctypes.data; s.dtype = DT[st[2]]
        elif name == "aux_load":
            arr = _check(st[1], st[2]); keep.append(arr)
            s.ptr = arr.ctypes.data; s.dtype = DT[st[2]]
            s.ld = arr.shape[-1]
            s.p0 = float(st[3]) if len(st) > 3 else 1.0
        elif name == "aux_store":
            arr = _check(st[1], "f64"); keep.append(arr)
            s.ptr = arr.ctypes.data; s.dtype = DT[st[2]]
            s.ld = arr.shape[-1]
    return c


def _rows(rows):
    if rows is None:
        return None, 0, None
    r = np.ascontiguousarray(rows, dtype=np.int64)
    return _ptr(r), len(r), r


def gemm(A, dtA, a_strides, B, dtB, b_strides, M, N, K, chain=None, rows=None, want_abs=False):
    """D[m,n] = E(sum_k A[m*a_rs + k*a_cs] * B[k*b_rs + n*b_cs]); returns float64 [M or len(rows), N]."""
    keep = []
    _check(A, dtA); _check(B, dtB)
    c = _chain(chain, keep)
    rp, nr, rk = _rows(rows)
    R = nr if rows is not None else M
    D = np.empty((R, N), dtype=np.float64)
    S = np.empty((R, N), dtype=np.float64) if want_abs else None
    lib().orc_gemm(C.c_int64(M), C.c_int64(N), C.c_int64(K),
                   _ptr(A), DT[dtA], C.c_int64(a_strides[0]), C.c_int64(a_strides[1]),
                   _ptr(B), DT[dtB], C.c_int64(b_strides[0]), C.c_int64(b_strides[1]),
                   C.byref(c) if c is not None else None, rp, C.c_int64(nr),
                   _ptr(D), _ptr(S) if want_abs else None)
    return (D, S) if want_abs else D


def batched_gemm(A, dtA, a_strides, B, dtB, b_strides, batch, M, N, K, chain=None,
                 aux_bs=0, want_abs=False):
    """a_strides / b_strides = (row, col, batch) element strides; returns [batch, M, N]."""
    keep = []
    _check(A, dtA); _check(B, dtB)
    c = _chain(chain, keep)
    D = np.empty((batch, M, N), dtype=np.float64)
    S = np.empty((batch, M, N), dtype=np.float64) if want_abs else None
    lib().orc_batched_gemm(C.c_int64(batch), C.c_int64(M), C.c_int64(N), C.c_int64(K),
                           _ptr(A), DT[dtA], *(C.c_int64(s) for s in a_strides),
                           _ptr(B), DT[dtB], *(C.c_int64(s) for s in b_strides),
                           C.byref(c) if c is not None else None, C.c_int64(aux_bs),
                           _ptr(D), _ptr(S) if want_abs else None)
    return (D, S) if want_abs else D


def grouped_gemm(A_list, dtA, a_strides, B_list, dtB, b_strides, M_g, N, K, chains=None,
                 want_abs=False):
    """Per-group operands as lists of arrays; chains = None or one chain per group.
    Returns the packed [sum M_g, N] result."""
    G = len(M_g)
    keep = []
    Mg = np.asarray(M_g, dtype=np.int64)
    Ap = (C.c_void_p * G)(*[a.ctypes.data for a in A_list])
    Bp = (C.c_void_p * G)(*[b.ctypes.data for b in B_list])
    for a in A_list:
        _check(a, dtA)
    for b in B_list:
        _check(b, dtB)
    carr = None
    if chains is not None:
        carr = (_Chain * G)()
        for g in range(G):
            cg = _chain(chains[g], keep)
            if cg is not None:
                carr[g] = cg
    tot = int(Mg.sum())
    D = np.empty((tot, N), dtype=np.float64)
    S = np.empty((tot, N), dtype=np.float64) if want_abs else None
    lib().orc_grouped_gemm(C.c_int32(G), _ptr(Mg), C.c_int64(N), C.c_int64(K),
                           Ap, DT[dtA], C.c_int64(a_strides[0]), C.c_int64(a_strides[1]),
                           Bp, DT[dtB], C.c_int64(b_strides[0]), C.c_int64(b_strides[1]),
                           carr, _ptr(D), _ptr(S) if want_abs else None)
    return (D, S) if want_abs else D


def conv_out_dim(inp, pad, dil, ker, stride):
    return int(lib().orc_conv_out_dim(inp, pad, dil, ker, stride))


def conv2d_fprop(x, dtX, w, dtW, Nb, H, W, Cin, Ko, R, S, pad=(0, 0), stride=(1, 1), dil=(1, 1),
                 chain=None, rows=None, want_abs=False):
    """x NHWC, w KRSC -> y as a [Nb*P*Q (or len(rows)), Ko] float64 matrix."""
    keep = []
    _check(x, dtX); _check(w, dtW)
    c = _chain(chain, keep)
    P = conv_out_dim(H, pad[0], dil[0], R, stride[0])
    Q = conv_out_dim(W, pad[1], dil[1], S, stride[1])
    rp, nr, rk = _rows(rows)
    total = nr if rows is not None else Nb * P * Q
    D = np.empty((total, Ko), dtype=np.float64)
    Sabs = np.empty((total, Ko), dtype=np.float64) if want_abs else None
    lib().orc_conv2d_fprop(*(C.c_int64(v) for v in (Nb, H, W, Cin, Ko, R, S, pad[0], pad[1],
                                                    stride[0], stride[1], dil[0], dil[1])),
                           _ptr(x), DT[dtX], _ptr(w), DT[dtW],
                           C.byref(c) if c is not None else None, rp, C.c_int64(nr),
                           _ptr(D), _ptr(Sabs) if want_abs else None)
    return (D, Sabs) if want_abs else D


def conv2d_dgrad(dy, dtY, w, dtW, Nb, H, W, Cin, Ko, R, S, pad=(0, 0), stride=(1, 1), dil=(1, 1),
                 chain=None, rows=None, want_abs=False):
    """dy NPQK (P, Q as fprop gives them for this geometry), w KRSC -> dx as a [Nb*H*W (or len(rows)), Cin]
    float64 matrix (grammar `conv2d_dgrad`)."""
    keep = []
    _check(dy, dtY); _check(w, dtW)
    c = _chain(chain, keep)
    rp, nr, rk = _rows(rows)
    total = nr if rows is not None else Nb * H * W
    D = np.empty((total, Cin), dtype=np.float64)
    Sabs = np.empty((total, Cin), dtype=np.float64) if want_abs else None
    lib().orc_conv2d_dgrad(*(C.c_int64(v) for v in (Nb, H, W, Cin, Ko, R, S, pad[0], pad[1],
                                                    stride[0], stride[1], dil[0], dil[1])),
                           _ptr(dy), DT[dtY], _ptr(w), DT[dtW],
                           C.byref(c) if c is not None else None, rp, C.c_int64(nr),
                           _ptr(D), _ptr(Sabs) if want_abs else None)
    return (D, Sabs) if want_abs else D


def conv2d_wgrad(dy, dtY, x, dtX, Nb, H, W, Cin, Ko, R, S, pad=(0, 0), stride=(1, 1), dil=(1, 1),
                 chain=None, rows=None, want_abs=False):
    """dy NPQK, x NHWC -> dw as a [Ko (or len(rows)), R*S*Cin] float64 matrix, i.e. KRSC
    (grammar `conv2d_wgrad`)."""
    keep = []
    _check(dy, dtY); _check(x, dtX)
    c = _chain(chain, keep)
    rp, nr, rk = _rows(rows)
    total = nr if rows is not None else Ko
    D = np.empty((total, R * S * Cin), dtype=np.float64)
    Sabs = np.empty((total, R * S * Cin), dtype=np.float64) if want_abs else None
    lib().orc_conv2d_wgrad(*(C.c_int64(v) for v in (Nb, H, W, Cin, Ko, R, S, pad[0], pad[1],
                                                    stride[0], stride[1], dil[0], dil[1])),
                           _ptr(dy), DT[dtY], _ptr(x), DT[dtX],
                           C.byref(c) if c is not None else None, rp, C.c_int64(nr),
                           _ptr(D), _ptr(Sabs) if want_abs else None)
    return (D, Sabs) if want_abs else D


def transpose(src, dtype, batch, rows, cols):
    """dst[b][c][r] = src[b][r][c] as unrounded float64 (grammar `transpose_op`); round_to() gives
    what the target type stores."""
    _check(src, dtype)
    assert src.size == batch * rows * cols
    out = np.empty((batch, cols, rows), dtype=np.float64)
    if out.size:
        lib().orc_transpose(C.c_int64(batch), C.c_int64(rows), C.c_int64(cols), _ptr(src), DT[dtype], _ptr(out))
    return out


def epilogue(v, m, n, chain):
    keep = []
    c = _chain(chain, keep)
    return float(lib().orc_epilogue(float(v), m, n, C.byref(c) if c is not None else None))


def round_to(x, dtype):
    """Value that format `dtype` stores for x (round to nearest, ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    lib().orc_round_array(_ptr(x), _ptr(y), C.c_int64(x.size), DT[dtype])
    return y


def load(arr, dtype):
    """Decode stored bit patterns to float64, element by element."""
    _check(arr, dtype)
    flat = arr.reshape(-1)
    out = np.empty(flat.size, dtype=np.float64)
    L = lib()
    for i in range(flat.size):
        out[i] = L.orc_load(_ptr(flat), DT[dtype], i)
    return out.reshape(arr.shape)


def encode16(x, dtype):
    return int(lib().orc_encode16(float(x), DT[dtype]))


def sol_bound(flops, nbytes, peak_flops_at_max, compute_clock_ratio, peak_bw_at_max,
              mem_clock_ratio=1.0):
    s = _Sol()
    lib().orc_sol_bound(flops, nbytes, peak_flops_at_max, compute_clock_ratio, peak_bw_at_max,
                        mem_clock_ratio, C.byref(s))
    return {k: getattr(s, k) for k, _ in _Sol._fields_ if k != "pad_"}


def gemm_flops(batch, M, N, K):
    return float(lib().orc_gemm_flops(batch, M, N, K))
