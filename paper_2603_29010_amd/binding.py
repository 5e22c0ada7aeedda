"""ctypes binding of include/ucl.h -- argument marshalling only, same names as the C entry points.

Device buffers are passed as integer addresses (``tensor.data_ptr()``); nothing here touches
their contents.  A nonzero status raises UclError carrying ucl_last_error().
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libucl.so")

DTYPES = {"f32": 0, "f16": 1, "bf16": 2, "e4m3": 3, "e5m2": 4}
EPI_OPS = {
    "scale": 1, "bias": 2, "aux_load": 3, "relu": 4, "gelu_tanh": 5, "gelu_erf": 6, "silu": 7,
    "sigmoid": 8, "tanh": 9, "mish": 10, "hardswish": 11, "leaky_relu": 12, "elu": 13, "clamp": 14,
    "per_row_scale": 15, "per_col_scale": 16, "row_broadcast": 17, "column_broadcast": 18,
    "aux_store": 19,
}
OP_KINDS = {"gemm": 0, "batched_gemm": 1, "grouped_gemm": 2, "conv2d_fprop": 3, "conv2d_dgrad": 4, "conv2d_wgrad": 5}
MAX_EPI_STEPS = 8


class UclError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{status}: {message}")
        self.status = status
        self.message = message


class _EpiStep(C.Structure):
    _fields_ = [("op", C.c_int32), ("dtype", C.c_int32), ("p0", C.c_float), ("p1", C.c_float),
                ("ptr", C.c_void_p), ("ld", C.c_int64), ("bs", C.c_int64)]


class _Epilogue(C.Structure):
    _fields_ = [("n_steps", C.c_int32), ("reserved", C.c_int32), ("steps", _EpiStep * MAX_EPI_STEPS)]


class _Tuning(C.Structure):
    _fields_ = [("tile_m", C.c_int32), ("tile_n", C.c_int32), ("tile_k", C.c_int32),
                ("stages", C.c_int32), ("raster", C.c_int32), ("iterator", C.c_int32),
                ("split_k_mode", C.c_int32), ("split_k_slices", C.c_int32), ("scheduler", C.c_int32),
                ("reserved", C.c_int32), ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64)]


SPLIT_K_MODES = {"none": 0, "serial": 1, "parallel": 2}
SCHEDULERS = {"default": 0, "persistent": 1, "stream_k": 2}
WORKSPACE_COUNTER_BYTES = 65536
STATIC_WORKSPACE_BYTES = WORKSPACE_COUNTER_BYTES + (8 << 20)


class _Problem(C.Structure):
    _fields_ = [("op", C.c_int32), ("dt_in", C.c_int32), ("dt_out", C.c_int32), ("groups", C.c_int32),
                ("batch", C.c_int64), ("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64),
                ("M_g", C.POINTER(C.c_int64)),
                ("cN", C.c_int64), ("cH", C.c_int64), ("cW", C.c_int64), ("cC", C.c_int64),
                ("cKout", C.c_int64), ("cR", C.c_int64), ("cS", C.c_int64),
                ("pad_h", C.c_int64), ("pad_w", C.c_int64), ("stride_h", C.c_int64),
                ("stride_w", C.c_int64), ("dil_h", C.c_int64), ("dil_w", C.c_int64),
                ("epi", C.POINTER(_Epilogue)), ("a_layout", C.c_int32), ("b_layout", C.c_int32)]


class _VariantInfo(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("tile_m", "tile_n", "tile_k", "stages", "iterator", "op_class", "dt_in",
                                         "a_layout", "b_layout", "a_path", "b_path", "lds_bytes", "scheduler", "patch_channels")]


class _Hw(C.Structure):
    _fields_ = [("peak_flops_16bit", C.c_double), ("peak_flops_f32", C.c_double), ("peak_bw", C.c_double),
                ("compute_clock_ratio", C.c_double), ("memory_clock_ratio", C.c_double), ("peak_flops_8bit", C.c_double)]


class _SolReport(C.Structure):
    _fields_ = [("flops", C.c_double), ("bytes", C.c_double), ("peak_flops", C.c_double),
                ("peak_bw", C.c_double), ("ai", C.c_double), ("ridge", C.c_double),
                ("t_compute", C.c_double), ("t_mem", C.c_double), ("t_sol", C.c_double),
                ("compute_bound", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2603_29010_amd.build` "
                "(hipcc, gfx950). There is no fallback implementation.")
        # Device memory and streams come from PyTorch-ROCm, which ships its own copy of the HIP
        # runtime.  Import it first so that the process holds ONE runtime (the one that owns the
        # caller's allocations and streams) and libucl.so binds to it.
        import torch  # noqa: F401
        lib = C.CDLL(_LIB_PATH)
        i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
        lib.ucl_gemm.restype = C.c_int
        lib.ucl_gemm.argtypes = [i64, i64, i64, vp, i32, i64, i64, vp, i32, i64, i64, vp, i32, i64, i64,
                                 C.POINTER(_Epilogue), C.POINTER(_Tuning), vp]
        lib.ucl_gemm_static_workspace.restype = C.c_int
        lib.ucl_gemm_static_workspace.argtypes = lib.ucl_gemm.argtypes
        lib.ucl_batched_gemm.restype = C.c_int
        lib.ucl_batched_gemm.argtypes = [i64, i64, i64, i64, vp, i32, i64, i64, i64, vp, i32, i64, i64, i64,
                                         vp, i32, i64, i64, i64, C.POINTER(_Epilogue), C.POINTER(_Tuning), vp]
        lib.ucl_grouped_gemm.restype = C.c_int
        lib.ucl_grouped_gemm.argtypes = [i32, C.POINTER(i64), i64, i64, vp, i32, i64, i64, vp, i32, i64, i64,
                                         vp, i32, i64, i64, C.POINTER(_Epilogue), C.POINTER(_Tuning), vp]
        lib.ucl_conv2d_fprop.restype = C.c_int
        lib.ucl_conv2d_fprop.argtypes = [i64] * 13 + [vp, i32, vp, i32, vp, i32, C.POINTER(_Epilogue),
                                                      C.POINTER(_Tuning), vp]
        for fn in (lib.ucl_conv2d_dgrad, lib.ucl_conv2d_wgrad):
            fn.restype = C.c_int
            fn.argtypes = lib.ucl_conv2d_fprop.argtypes
        lib.ucl_transpose.restype = C.c_int
        lib.ucl_transpose.argtypes = [i64, i64, i64, vp, i32, vp, i32, vp]
        lib.ucl_sol_bound.restype = C.c_int
        lib.ucl_sol_bound.argtypes = [C.POINTER(_Problem), C.POINTER(_Hw), C.POINTER(_SolReport)]
        lib.ucl_select_tuning.restype = C.c_int
        lib.ucl_select_tuning.argtypes = [C.POINTER(_Problem), C.POINTER(_Tuning)]
        lib.ucl_workspace_size.restype = C.c_int
        lib.ucl_workspace_size.argtypes = [C.POINTER(_Problem), C.POINTER(_Tuning), C.POINTER(i64), C.POINTER(i32)]
        lib.ucl_workspace_init.restype = C.c_int
        lib.ucl_workspace_init.argtypes = [vp, i64, vp]
        lib.ucl_tile_map.restype = C.c_int
        lib.ucl_tile_map.argtypes = [i32, C.POINTER(i32), i32, i32, i32, C.POINTER(i32), C.POINTER(i32),
                                     C.POINTER(i32)]
        lib.ucl_num_variants.restype = i32
        lib.ucl_variant.restype = C.c_int
        lib.ucl_variant.argtypes = [i32, C.POINTER(_VariantInfo)]
        lib.ucl_status_string.restype = C.c_char_p
        lib.ucl_status_string.argtypes = [C.c_int]
        lib.ucl_last_error.restype = C.c_char_p
        lib.ucl_version.restype = C.c_char_p
        _lib = lib
    return _lib


def _check(st):
    if st != 0:
        lib = _load()
        raise UclError(lib.ucl_status_string(st).decode(), lib.ucl_last_error().decode())


def _dt(d):
    return DTYPES[d] if isinstance(d, str) else int(d)


class Epilogue:
    """Ordered `>>` chain.  steps: (name,), (name, p0[, p1]) or
    (name, ptr, dtype[, ld[, bs[, p0]]]) for ops with a tensor operand (ptr = device address)."""

    TENSOR = {"bias", "aux_load", "per_row_scale", "per_col_scale", "row_broadcast",
              "column_broadcast", "aux_store"}

    def __init__(self, steps=()):
        self.c = _Epilogue()
        if len(steps) > MAX_EPI_STEPS:
            raise UclError("UCL_ERR_INVALID_ARG", f"at most {MAX_EPI_STEPS} epilogue steps")
        self.c.n_steps = len(steps)
        for i, st in enumerate(steps):
            s = self.c.steps[i]
            name = st[0]
            s.op = EPI_OPS[name] if isinstance(name, str) else int(name)
            if name in self.TENSOR:
                s.ptr = int(st[1])
                s.dtype = _dt(st[2])
                s.ld = int(st[3]) if len(st) > 3 else 0
                s.bs = int(st[4]) if len(st) > 4 else 0
                s.p0 = float(st[5]) if len(st) > 5 else 1.0
            else:
                s.p0 = float(st[1]) if len(st) > 1 else 0.0
                s.p1 = float(st[2]) if len(st) > 2 else 0.0

    def ref(self):
        return C.byref(self.c)


class Tuning:
    """split_k: "none" | "serial" | "parallel" (or the enum value); workspace: device address."""

    def __init__(self, tile_m=0, tile_n=0, tile_k=0, stages=0, raster=0, iterator=0, split_k="none", slices=0,
                 scheduler="default", workspace=0, workspace_bytes=0):
        mode = SPLIT_K_MODES[split_k] if isinstance(split_k, str) else int(split_k)
        sched = SCHEDULERS[scheduler] if isinstance(scheduler, str) else int(scheduler)
        self.c = _Tuning(tile_m, tile_n, tile_k, stages, raster, iterator, mode, slices, sched, 0,
                         workspace or None, workspace_bytes)

    def ref(self):
        return C.byref(self.c)

    def as_dict(self):
        return {k: getattr(self.c, k) for k in ("tile_m", "tile_n", "tile_k", "stages", "raster", "iterator")}


def _opt(x):
    return x.ref() if x is not None else None


def ucl_gemm(M, N, K, A, dtA, a_rs, a_cs, B, dtB, b_rs, b_cs, D, dtD, d_rs, d_cs, epi=None, tune=None,
             stream=0):
    _check(_load().ucl_gemm(M, N, K, A, _dt(dtA), a_rs, a_cs, B, _dt(dtB), b_rs, b_cs, D, _dt(dtD), d_rs, d_cs,
                            _opt(epi), _opt(tune), stream or None))


def ucl_gemm_static_workspace(M, N, K, A, dtA, a_rs, a_cs, B, dtB, b_rs, b_cs, D, dtD, d_rs, d_cs, epi=None, tune=None,
                              stream=0):
    _check(_load().ucl_gemm_static_workspace(M, N, K, A, _dt(dtA), a_rs, a_cs, B, _dt(dtB), b_rs, b_cs, D, _dt(dtD),
                                             d_rs, d_cs, _opt(epi), _opt(tune), stream or None))


def ucl_batched_gemm(batch, M, N, K, A, dtA, a_rs, a_cs, a_bs, B, dtB, b_rs, b_cs, b_bs, D, dtD, d_rs, d_cs,
                     d_bs, epi=None, tune=None, stream=0):
    _check(_load().ucl_batched_gemm(batch, M, N, K, A, _dt(dtA), a_rs, a_cs, a_bs, B, _dt(dtB), b_rs, b_cs, b_bs,
                                    D, _dt(dtD), d_rs, d_cs, d_bs, _opt(epi), _opt(tune), stream or None))


def ucl_grouped_gemm(M_g, N, K, A_g, dtA, a_rs, a_cs, B_g, dtB, b_rs, b_cs, D_g, dtD, d_rs, d_cs, epi=None,
                     tune=None, stream=0):
    """M_g: host sequence of ints; A_g / B_g / D_g: device addresses of the pointer tables."""
    G = len(M_g)
    arr = (C.c_int64 * max(G, 1))(*[int(m) for m in M_g])
    _check(_load().ucl_grouped_gemm(G, arr, N, K, A_g, _dt(dtA), a_rs, a_cs, B_g, _dt(dtB), b_rs, b_cs, D_g,
                                    _dt(dtD), d_rs, d_cs, _opt(epi), _opt(tune), stream or None))


def ucl_conv2d_fprop(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, x, dtX, w, dtW,
                     y, dtY, epi=None, tune=None, stream=0):
    _check(_load().ucl_conv2d_fprop(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w,
                                    x, _dt(dtX), w, _dt(dtW), y, _dt(dtY), _opt(epi), _opt(tune), stream or None))


def ucl_conv2d_dgrad(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, dy, dtDy, w, dtW,
                     dx, dtDx, epi=None, tune=None, stream=0):
    _check(_load().ucl_conv2d_dgrad(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w,
                                    dy, _dt(dtDy), w, _dt(dtW), dx, _dt(dtDx), _opt(epi), _opt(tune), stream or None))


def ucl_conv2d_wgrad(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, dy, dtDy, x, dtX,
                     dw, dtDw, epi=None, tune=None, stream=0):
    _check(_load().ucl_conv2d_wgrad(N, H, W, Cin, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w,
                                    dy, _dt(dtDy), x, _dt(dtX), dw, _dt(dtDw), _opt(epi), _opt(tune), stream or None))


def ucl_transpose(batch, rows, cols, src, dt_src, dst, dt_dst, stream=0):
    _check(_load().ucl_transpose(batch, rows, cols, src, _dt(dt_src), dst, _dt(dt_dst), stream or None))


LAYOUTS = {"k": 0, "mn": 1}


def _problem(op, dt_in, dt_out, batch=1, M=0, N=0, K=0, M_g=None, conv=None, epi=None, a_layout="k", b_layout="k"):
    """a_layout / b_layout: "k" (operand contiguous along K: A row-major, B column-major) or "mn"."""
    p = _Problem()
    p.a_layout, p.b_layout = LAYOUTS[a_layout], LAYOUTS[b_layout]
    p.op = OP_KINDS[op]
    p.dt_in, p.dt_out = _dt(dt_in), _dt(dt_out)
    p.batch, p.M, p.N, p.K = batch, M, N, K
    keep = []
    if M_g is not None:
        arr = (C.c_int64 * len(M_g))(*[int(m) for m in M_g])
        keep.append(arr)
        p.M_g = C.cast(arr, C.POINTER(C.c_int64))
        p.groups = len(M_g)
    if conv is not None:
        (p.cN, p.cH, p.cW, p.cC, p.cKout, p.cR, p.cS, p.pad_h, p.pad_w, p.stride_h, p.stride_w, p.dil_h,
         p.dil_w) = [int(v) for v in conv]
    if epi is not None:
        p.epi = C.pointer(epi.c)
        keep.append(epi)
    return p, keep


def ucl_sol_bound(op, dt_in, dt_out, hw=None, **kw):
    """hw: None (MI355X nominal) or dict(peak_flops_16bit, peak_flops_f32, peak_bw,
    compute_clock_ratio, memory_clock_ratio).  Returns the report as a dict."""
    p, keep = _problem(op, dt_in, dt_out, **kw)
    h = None
    if hw is not None:
        h = _Hw(hw.get("peak_flops_16bit", 0.0), hw.get("peak_flops_f32", 0.0), hw["peak_bw"],
                hw.get("compute_clock_ratio", 1.0), hw.get("memory_clock_ratio", 1.0), hw.get("peak_flops_8bit", 0.0))
    r = _SolReport()
    _check(_load().ucl_sol_bound(C.byref(p), C.byref(h) if h is not None else None, C.byref(r)))
    return {k: getattr(r, k) for k, _ in _SolReport._fields_ if k != "reserved"}


def ucl_select_tuning(op, dt_in, dt_out, **kw):
    p, keep = _problem(op, dt_in, dt_out, **kw)
    t = Tuning()
    _check(_load().ucl_select_tuning(C.byref(p), t.ref()))
    return t.as_dict()


def ucl_workspace_size(op, dt_in, dt_out, tune=None, **kw):
    """(bytes, slices) a call on this problem with this tuning needs / uses."""
    p, keep = _problem(op, dt_in, dt_out, **kw)
    nbytes, slices = C.c_int64(), C.c_int32()
    _check(_load().ucl_workspace_size(C.byref(p), _opt(tune), C.byref(nbytes), C.byref(slices)))
    return nbytes.value, slices.value


def ucl_workspace_init(workspace, workspace_bytes, stream=0):
    _check(_load().ucl_workspace_init(workspace, workspace_bytes, stream or None))


def ucl_tile_map(tiles_m, tiles_n, raster, wg):
    G = len(tiles_m)
    arr = (C.c_int32 * G)(*tiles_m)
    g, tm, tn = C.c_int32(), C.c_int32(), C.c_int32()
    _check(_load().ucl_tile_map(G, arr, tiles_n, raster, wg, C.byref(g), C.byref(tm), C.byref(tn)))
    return g.value, tm.value, tn.value


def ucl_num_variants():
    return int(_load().ucl_num_variants())


def ucl_variant(i):
    """Variant i as a dict of the ucl_variant_info fields, plus the short keys the tests filter on:
    mode = op_class, f16 = 1 for fp16 inputs, la / lb = a_path / b_path."""
    v = _VariantInfo()
    _check(_load().ucl_variant(i, C.byref(v)))
    d = {k: getattr(v, k) for k, _ in _VariantInfo._fields_}
    d["mode"], d["f16"], d["la"], d["lb"] = v.op_class, int(v.dt_in == DTYPES["f16"]), v.a_path, v.b_path
    d["dt"] = {code: name for name, code in DTYPES.items()}[v.dt_in]
    return d


def ucl_last_error():
    return _load().ucl_last_error().decode()


def ucl_version():
    return _load().ucl_version().decode()
