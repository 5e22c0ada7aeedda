"""Seeded synthetic inputs for the five benchmark workloads and their scaled-down kin.

This module only *draws numbers and lays them out*; it holds none of the
arithmetic of the operations under test (no products, no epilogues), so both
the GPU library's tests and the CPU checker can be fed from it.

Generator: counter-based.  Element ``i`` of tensor ``t`` under seed ``s`` is a
function of ``(s, t, i)`` alone -- a SplitMix64-style finaliser over the packed
counter -- so any slice of any tensor can be regenerated independently of
allocation order or library version.  Uniform = top 53 bits * 2^-53; normal =
Box-Muller on two such draws.  Values are computed in float64 and rounded once
to the storage format; what both sides consume are the stored bit patterns
(``uint16`` for bf16 / fp16, ``float32`` for fp32).

A workload is a plain dict ("spec"):
  op        "gemm" | "batched_gemm" | "grouped_gemm" | "conv2d_fprop"
  dt_in, dt_out   "bf16" | "f16" | "f32"
  shapes    M,N,K (+batch / M_g / conv geometry)
  tensors   numpy arrays of stored bits, plus element strides
  epilogue  list of steps, each (name, *args) with tensor operands named by key
"""
import math

import numpy as np

BASE_SEED = 260329010
_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z):
    """SplitMix64 finaliser, vectorised over uint64 (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + np.uint64(0x9E3779B97F4A7C15)) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        return z ^ (z >> np.uint64(31))


def raw_u64(seed, tensor_id, start, count, stream=0):
    """Hash of (seed, tensor, stream, index) for index in [start, start+count)."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * np.uint64(0x100000001B3) + np.uint64(tensor_id) * np.uint64(0x9E37)
                   + np.uint64(stream))
        return _mix(idx ^ key)


def uniform01(seed, tensor_id, n, stream=0, start=0):
    """float64 in [0, 1)."""
    return (raw_u64(seed, tensor_id, start, n, stream) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53


def uniform_pm1(seed, tensor_id, n):
    return 2.0 * uniform01(seed, tensor_id, n) - 1.0


def normal(seed, tensor_id, n):
    u1 = uniform01(seed, tensor_id, n, stream=1) + 2.0 ** -53      # (0, 1]
    u2 = uniform01(seed, tensor_id, n, stream=2)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def randint(seed, tensor_id, n, lo, hi):
    """Integers uniform on [lo, hi] (inclusive), as float64."""
    span = np.uint64(hi - lo + 1)
    return (raw_u64(seed, tensor_id, 0, n, stream=3) % span).astype(np.float64) + lo


# ---- storage formats -------------------------------------------------------------------------

def to_bits(x, dtype):
    """Round float64 values once (ties to even) to `dtype` and return the stored array."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype in ("e4m3", "e5m2"):
        # the library cast (ties to even, e4m3 saturating at +-448); values are kept inside the finite range
        import torch
        t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
        lim = 448.0 if dtype == "e4m3" else 57344.0
        t = t.clamp(-lim, lim).to(torch.float8_e4m3fn if dtype == "e4m3" else torch.float8_e5m2)
        return t.view(torch.uint8).numpy().copy()
    if dtype == "bf16":
        # float64 -> float32 -> bf16, each step ties-to-even.  (Two roundings; harmless here:
        # the stored bits *are* the input, nobody compares them to the float64 draw.)
        y = _bf16_via_f32(x.astype(np.float32))
        return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def _bf16_via_f32(f32):
    u = f32.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bits_to_f64(a, dtype):
    """Exact float64 value of stored bits (for building torch tensors / test bookkeeping only)."""
    if dtype == "f32":
        return a.astype(np.float64)
    if dtype == "f16":
        return a.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype in ("e4m3", "e5m2"):
        import torch
        t = torch.from_numpy(np.ascontiguousarray(a)).view(torch.float8_e4m3fn if dtype == "e4m3" else torch.float8_e5m2)
        return t.to(torch.float64).numpy()
    raise ValueError(dtype)


def itemsize(dtype):
    return {"e4m3": 1, "e5m2": 1, "bf16": 2, "f16": 2, "f32": 4}[dtype]


# ---- workloads -------------------------------------------------------------------------------

def gemm_spec(M, N, K, dt_in="bf16", dt_out="bf16", a_layout="row", b_layout="col",
              dist="normal", scale=None, epilogue=("bias", "relu"), seed=BASE_SEED, integer=False):
    """Dense GEMM.  a_layout "row": A stored [M,K]; "col": stored [K,M].
    b_layout "col": B stored [N,K] (K contiguous); "row": stored [K,N]."""
    if scale is None:
        scale = 1.0 / math.sqrt(K) if dist == "normal" else 1.0

    def draw(tid, n):
        if integer:
            return randint(seed, tid, n, -2, 2)
        return (normal(seed, tid, n) if dist == "normal" else uniform_pm1(seed, tid, n)) * scale

    A = to_bits(draw(1, M * K), dt_in).reshape((M, K) if a_layout == "row" else (K, M))
    B = to_bits(draw(2, N * K), dt_in).reshape((N, K) if b_layout == "col" else (K, N))
    spec = {
        "op": "gemm", "M": M, "N": N, "K": K, "dt_in": dt_in, "dt_out": dt_out,
        "A": A, "a_strides": (K, 1) if a_layout == "row" else (1, M),
        "B": B, "b_strides": (1, K) if b_layout == "col" else (N, 1),
        "tensors": {}, "epilogue": [],
    }
    _add_epilogue(spec, epilogue, draw, M, N, dt_out)
    return spec


def _add_epilogue(spec, names, draw, M, N, aux_dt, tid0=10, aux_rows=None, groups=None):
    """Attach epilogue steps; tensor operands are drawn like the main operands.
    aux_rows: row count of full-shape (aux_load) operands when it differs from M (batched).
    groups: grouped GEMM -- every group gets its own n-indexed vector, stored as row g of a
    [groups, N rounded up to 8] array (so that each row starts 16-byte aligned); m-indexed vectors
    and matrices are packed like the output, M = sum of the group sizes."""
    tid = tid0
    aux_rows = M if aux_rows is None else aux_rows
    for st in names:
        if isinstance(st, str):
            st = (st,)
        name = st[0]
        if name in ("bias", "per_col_scale", "row_broadcast"):
            key = f"{name}{tid}"
            if groups is None:
                spec["tensors"][key] = (to_bits(draw(tid, N), aux_dt), aux_dt)
            else:
                npad = (N + 7) // 8 * 8
                spec["tensors"][key] = (to_bits(draw(tid, groups * npad), aux_dt).reshape(groups, npad), aux_dt)
            spec["epilogue"].append((name, key))
        elif name in ("per_row_scale", "column_broadcast"):
            key = f"{name}{tid}"
            spec["tensors"][key] = (to_bits(draw(tid, M), aux_dt), aux_dt)
            spec["epilogue"].append((name, key))
        elif name == "aux_load":
            key = f"{name}{tid}"
            spec["tensors"][key] = (to_bits(draw(tid, aux_rows * N), aux_dt).reshape(aux_rows, N), aux_dt)
            spec["epilogue"].append((name, key) + tuple(st[1:]))
        else:
            spec["epilogue"].append(tuple(st))
        tid += 1


def batched_spec(batch, M, N, K, dt_in="f16", dt_out="f32", scale=1.0, epilogue=None,
                 seed=BASE_SEED + 3, integer=False, a_layout="row", b_layout="col"):
    """Strided batched GEMM, A stored [b,M,K], B stored [b,N,K] (Q.K^T-like), D [b,M,N];
    a_layout="col" stores A as [b,K,M], b_layout="row" stores B as [b,K,N] (P.V-like)."""
    def draw(tid, n):
        if integer:
            return randint(seed, tid, n, -2, 2)
        return normal(seed, tid, n) * scale

    A = to_bits(draw(1, batch * M * K), dt_in).reshape((batch, M, K) if a_layout == "row" else (batch, K, M))
    B = to_bits(draw(2, batch * N * K), dt_in).reshape((batch, N, K) if b_layout == "col" else (batch, K, N))
    spec = {
        "op": "batched_gemm", "batch": batch, "M": M, "N": N, "K": K, "dt_in": dt_in, "dt_out": dt_out,
        "A": A, "a_strides": (K, 1, M * K) if a_layout == "row" else (1, M, M * K),
        "B": B, "b_strides": (1, K, N * K) if b_layout == "col" else (N, 1, N * K),
        "tensors": {}, "epilogue": [],
    }
    if epilogue is None:
        epilogue = [("scale", 1.0 / math.sqrt(K))]
    _add_epilogue(spec, epilogue, draw, M, N, dt_out, aux_rows=batch * M)
    return spec


def grouped_sizes(groups, seed, lo=128, step=64, count=31):
    """M_i = lo + step*j with j uniform on {0..count-1}, independent per group."""
    j = (raw_u64(seed, 99, 0, groups, stream=7) % np.uint64(count)).astype(np.int64)
    return [int(lo + step * v) for v in j]


def grouped_spec(M_g, N, K, dt_in="bf16", dt_out="bf16", scale=None, epilogue=("silu",),
                 seed=BASE_SEED + 4, integer=False, b_layout="col"):
    """Grouped GEMM: A packed [sum M_g, K] (row-major), one B per group stored [N,K] (column-major B,
    the default) or [K,N] (b_layout="row"), D packed.  Epilogue tensors are per group: a [G, N]
    array of n-indexed vectors, m-indexed vectors and matrices packed like D."""
    if scale is None:
        scale = 1.0 / math.sqrt(K)
    G = len(M_g)
    tot = int(sum(M_g))

    def draw(tid, n):
        if integer:
            return randint(seed, tid, n, -2, 2)
        return normal(seed, tid, n) * scale

    A = to_bits(draw(1, tot * K), dt_in).reshape(tot, K)
    row = b_layout == "row"
    B = to_bits(draw(2, G * N * K), dt_in).reshape((G, K, N) if row else (G, N, K))
    spec = {
        "op": "grouped_gemm", "M_g": list(M_g), "N": N, "K": K, "dt_in": dt_in, "dt_out": dt_out,
        "A": A, "a_strides": (K, 1), "B": B, "b_strides": (N, 1) if row else (1, K),
        "tensors": {}, "epilogue": [],
    }
    _add_epilogue(spec, epilogue, draw, tot, N, dt_out, groups=G)
    return spec


def conv_spec(Nb, H, W, C, Ko, R, S, pad=(1, 1), stride=(1, 1), dil=(1, 1), dt_in="bf16",
              dt_out="bf16", scale=None, epilogue=("bias", "aux_load", "relu"),
              seed=BASE_SEED + 5, integer=False):
    """conv2d forward, x NHWC, w KRSC, y NPQK."""
    if scale is None:
        scale = 1.0 / math.sqrt(R * S * C)

    def draw(tid, n):
        if integer:
            return randint(seed, tid, n, -2, 2)
        return normal(seed, tid, n) * scale

    P = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    x = to_bits(draw(1, Nb * H * W * C), dt_in).reshape(Nb, H, W, C)
    w = to_bits(draw(2, Ko * R * S * C), dt_in).reshape(Ko, R, S, C)
    spec = {
        "op": "conv2d_fprop", "Nb": Nb, "H": H, "W": W, "C": C, "Ko": Ko, "R": R, "S": S,
        "P": P, "Q": Q, "pad": tuple(pad), "stride": tuple(stride), "dil": tuple(dil),
        "dt_in": dt_in, "dt_out": dt_out, "x": x, "w": w, "tensors": {}, "epilogue": [],
        "M": Nb * P * Q, "N": Ko, "K": R * S * C,
    }
    _add_epilogue(spec, epilogue, draw, Nb * P * Q, Ko, dt_out)
    return spec


def conv_grad_spec(kind, Nb, H, W, C, Ko, R, S, pad=(1, 1), stride=(1, 1), dil=(1, 1), dt_in="bf16",
                   dt_out="bf16", scale=None, epilogue=(), seed=BASE_SEED + 7, integer=False):
    """conv2d_dgrad (kind "dgrad": dy NPQK, w KRSC -> dx NHWC) or conv2d_wgrad (kind "wgrad": dy NPQK,
    x NHWC -> dw KRSC) of the forward geometry given.  M, N, K are those of the implicit GEMM."""
    P = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    if kind == "dgrad":
        M, N, K = Nb * H * W, C, R * S * Ko
    else:
        M, N, K = Ko, R * S * C, Nb * P * Q
    if scale is None:
        scale = 1.0 / math.sqrt(math.sqrt(K))      # both factors scaled: products of variance 1/K

    def draw(tid, n):
        if integer:
            return randint(seed, tid, n, -2, 2)
        return normal(seed, tid, n) * scale

    spec = {
        "op": "conv2d_" + kind, "Nb": Nb, "H": H, "W": W, "C": C, "Ko": Ko, "R": R, "S": S, "P": P, "Q": Q,
        "pad": tuple(pad), "stride": tuple(stride), "dil": tuple(dil), "dt_in": dt_in, "dt_out": dt_out,
        "dy": to_bits(draw(1, Nb * P * Q * Ko), dt_in).reshape(Nb, P, Q, Ko),
        "tensors": {}, "epilogue": [], "M": M, "N": N, "K": K,
    }
    if kind == "dgrad":
        spec["w"] = to_bits(draw(2, Ko * R * S * C), dt_in).reshape(Ko, R, S, C)
    else:
        spec["x"] = to_bits(draw(2, Nb * H * W * C), dt_in).reshape(Nb, H, W, C)
    _add_epilogue(spec, epilogue, draw, M, N, dt_out)
    return spec


def config(i, shrink=1):
    """The five benchmark workloads (i = 1..5).  shrink > 1 divides the large extents so the
    CPU checker finishes quickly while the structure (layouts, epilogue, raggedness) is kept."""
    s = shrink
    if i == 1:
        return gemm_spec(256, 256, 256, a_layout="row", b_layout="row", dist="uniform",
                         epilogue=("bias", "relu"), seed=BASE_SEED + 1)
    if i == 2:
        n = 4096 // s
        return gemm_spec(n, n, n, a_layout="row", b_layout="col", dist="normal", scale=1.0 / 64,
                         epilogue=("bias", "gelu_tanh"), seed=BASE_SEED + 2)
    if i == 3:
        return batched_spec(64 // s, 512, 512, 128, seed=BASE_SEED + 3)
    if i == 4:
        M_g = grouped_sizes(16, BASE_SEED + 4)
        if s > 1:
            M_g = [max(64, (m // s) // 64 * 64) for m in M_g]
        return grouped_spec(M_g, 4096 // s, 1024 // s if s > 1 else 1024, scale=1.0 / 32,
                            seed=BASE_SEED + 4)
    if i == 5:
        return conv_spec(32 // s, 56, 56, 64, 128, 3, 3, scale=1.0 / 24, seed=BASE_SEED + 5)
    raise ValueError(i)
