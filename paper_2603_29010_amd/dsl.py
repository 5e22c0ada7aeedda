"""Host-side translator from the kernel DSL's text to calls of the C ABI.

The paper's DSL (Sec. 3; appendix "Full EBNF Grammar") writes a kernel as an operation, a list of
`.with_*` configuration calls and a `>>` chain of epilogue operations, or several such stages inside
`pipeline(...)`.  This module parses that text with a small recursive-descent parser written for the
grammar's rules (start, kernel, pipeline, stage, transpose_op, operation, configuration, epilogue_op)
and lowers the result to what `ucl_*` takes: entry point, dtype codes, operand strides, `ucl_tuning`,
the ordered `ucl_epilogue` steps.  It computes nothing: `launch()` marshals and calls the library.

What is lowered and what is not
  * operations: gemm, batched_gemm, grouped_gemm, conv2d_fprop / dgrad / wgrad, conv1d_fprop (as H = 1);
    transpose stages.  conv3d, depthwise and group convolutions are parsed and rejected with a reason.
  * `.with_dtype`: input fp16 | bf16 | fp8_e4m3 | fp8_e5m2, acc fp32, output fp16 | bf16 | fp32.
  * `.with_layout`, `.with_tile` / `.with_threadblockshape`, `.with_stages`, `.with_alignment` (checked
    against the grammar's rule (alignment * element_size) % 16 == 0), `.with_swizzle`, `.with_scaling`,
    `.with_iterator`, `.with_split_k`, `.with_scheduler(tile=..., splits=...)`.
  * `.with_arch`, `.with_cluster`, `.with_operand_swap` and the kernel= / epilogue= schedules of
    `.with_scheduler` name NVIDIA hardware features; they are accepted, recorded in `Kernel.ignored`
    and have no effect (the library is built for one architecture).
  * every epilogue_op except custom('...'); gelu() lowers to the erf form unless gelu="tanh" is given.
"""
import math
import re

from . import binding as ucl


class DslError(ValueError):
    """A program the grammar or the library's limits reject; the message says what and why."""


# ---------------------------------------------------------------------------------- tokens

_TOKEN = re.compile(r"""
    (?P<ws>\s+|\#[^\n]*|\(\*.*?\*\))           |
    (?P<shift>>>)                                |
    (?P<num>-?\d+(?:\.\d+)?(?:[eE][-+]?\d+)?)    |
    (?P<str>'[^']*')                             |
    (?P<id>[A-Za-z_][A-Za-z_0-9]*)               |
    (?P<punct>[().,=:{}])
""", re.X | re.S)


def _tokens(text):
    out, pos = [], 0
    while pos < len(text):
        m = _TOKEN.match(text, pos)
        if not m:
            raise DslError(f"unexpected character {text[pos]!r} at offset {pos}")
        pos = m.end()
        kind = m.lastgroup
        if kind != "ws":
            out.append((kind, m.group(kind), m.start()))
    out.append(("end", "", len(text)))
    return out


# ---------------------------------------------------------------------------------- syntax tree

class Call:
    """name(arg, key=value, ...): positional values and keyword values as parsed."""

    def __init__(self, name, args, kwargs, pos):
        self.name, self.args, self.kwargs, self.pos = name, args, kwargs, pos

    def __repr__(self):
        parts = [repr(a) for a in self.args] + [f"{k}={v!r}" for k, v in self.kwargs.items()]
        return f"{self.name}({', '.join(parts)})"


class _Parser:
    def __init__(self, text):
        self.t = _tokens(text)
        self.i = 0

    def peek(self, k=0):
        return self.t[self.i + k]

    def take(self, kind=None, value=None):
        tok = self.t[self.i]
        if (kind and tok[0] != kind) or (value is not None and tok[1] != value):
            want = value if value is not None else kind
            raise DslError(f"expected {want!r} at offset {tok[2]}, found {tok[1]!r}")
        self.i += 1
        return tok

    def value(self):
        kind, v, pos = self.peek()
        if kind == "num":
            self.i += 1
            return float(v) if any(c in v for c in ".eE") else int(v)
        if kind == "str":
            self.i += 1
            return v[1:-1]
        if kind == "id":
            self.i += 1
            return v
        if kind == "punct" and v == "{":
            return self.dict_()
        raise DslError(f"expected a value at offset {pos}, found {v!r}")

    def dict_(self):
        self.take("punct", "{")
        d = {}
        while True:
            k = self.take("str")[1][1:-1]
            self.take("punct", ":")
            d[k] = self.take("str")[1][1:-1]
            if self.peek()[1] == ",":
                self.i += 1
                continue
            self.take("punct", "}")
            return d

    def call(self):
        kind, name, pos = self.take("id")
        self.take("punct", "(")
        args, kwargs = [], {}
        while self.peek()[1] != ")":
            if self.peek()[0] == "id" and self.peek(1)[1] == "=":
                key = self.take("id")[1]
                self.take("punct", "=")
                if key in kwargs:
                    raise DslError(f"{name}(): argument {key!r} given twice")
                kwargs[key] = self.value()
            else:
                args.append(self.value())
            if self.peek()[1] == ",":
                self.i += 1
        self.take("punct", ")")
        return Call(name, args, kwargs, pos)

    def kernel(self):
        op = self.call()
        configs, chain = [], []
        while self.peek()[1] == ".":
            self.i += 1
            configs.append(self.call())
        while self.peek()[0] == "shift":
            self.i += 1
            chain.append(self.call())
        if self.peek()[1] == ".":
            raise DslError(f"configuration after the epilogue chain at offset {self.peek()[2]}: the grammar puts every .with_* before the first >>")
        return Kernel(op, configs, chain)

    def program(self):
        if self.peek()[1] == "pipeline" and self.peek(1)[1] == "(":
            self.i += 2
            stages = []
            while True:
                if self.peek()[1] == "transpose":
                    stages.append(Transpose(self.call()))
                else:
                    stages.append(self.kernel())
                if self.peek()[1] == ",":
                    self.i += 1
                    continue
                break
            self.take("punct", ")")
            prog = Pipeline(stages)
        else:
            prog = self.kernel()
        self.take("end")
        return prog


# ---------------------------------------------------------------------------------- lowering tables

_DTYPES = {"fp32": "f32", "float32": "f32", "fp16": "f16", "float16": "f16", "bf16": "bf16", "bfloat16": "bf16",
           "fp8_e4m3": "e4m3", "e4m3": "e4m3", "fp8_e5m2": "e5m2", "e5m2": "e5m2"}
_KNOWN_DTYPES = set(_DTYPES) | {"fp64", "float64", "tf32", "int8", "s8", "int16", "s16", "int32", "s32", "uint8", "u8",
                                "uint16", "u16", "uint32", "u32"}
_ELEM_BYTES = {"f32": 4, "f16": 2, "bf16": 2, "e4m3": 1, "e5m2": 1}
_OPS = {"gemm": "gemm", "batched_gemm": "batched_gemm", "grouped_gemm": "grouped_gemm", "conv2d_fprop": "conv2d_fprop",
        "conv2d_dgrad": "conv2d_dgrad", "conv2d_wgrad": "conv2d_wgrad", "conv1d_fprop": "conv2d_fprop"}
_NOT_BUILT_OPS = {"depthwise_conv1d", "group_conv1d", "conv3d_fprop", "conv3d_dgrad", "conv3d_wgrad", "depthwise_conv2d",
                  "group_conv2d", "group_conv3d"}
_SIMPLE_ACT = {"relu": "relu", "silu": "silu", "mish": "mish", "sigmoid": "sigmoid", "tanh": "tanh", "hardswish": "hardswish"}
_SWIZZLE = {"Identity1": 1, "Identity2": 2, "Identity4": 4, "Identity8": 8}
_ITERATORS = {"analytic": 1, "optimized": 0, "fixed_stride_dilation": 2}
_NVIDIA_ONLY = {"with_arch", "with_cluster", "with_operand_swap"}


class Kernel:
    """One kernel stage: `op`, the `.with_*` calls and the `>>` chain, checked and lowered on construction."""

    def __init__(self, op, configs, chain, gelu="erf"):
        self.op_call, self.config_calls, self.chain_calls = op, configs, chain
        self.ignored = []                  # NVIDIA-specific settings that were accepted and have no effect
        self.gelu = gelu
        self._lower()

    # -- configuration --------------------------------------------------------------------------
    def _lower(self):
        name = self.op_call.name
        if name in _NOT_BUILT_OPS:
            raise DslError(f"{name}: parsed, but this library builds gemm, batched_gemm, grouped_gemm, conv2d_fprop / dgrad / wgrad and conv1d_fprop only")
        if name not in _OPS:
            raise DslError(f"unknown operation {name!r}")
        self.op = _OPS[name]
        self.is_conv = self.op.startswith("conv2d")
        kw = self.op_call.kwargs
        self.expert_count = None
        self.filter = None
        if name == "grouped_gemm":
            self.expert_count = self._int(kw, "expert_count", name)
        elif name == "conv1d_fprop":
            self.filter = (1, self._int(kw, "kernel_w", name))          # lowered to 2-D with H = 1 (Table "coverage")
        elif self.is_conv:
            self.filter = (self._int(kw, "kernel_h", name), self._int(kw, "kernel_w", name))
        elif kw or self.op_call.args:
            raise DslError(f"{name}() takes no arguments")
        seen = {}
        for c in self.config_calls:
            key = "with_tile" if c.name == "with_threadblockshape" else c.name
            if key in seen:
                raise DslError(f".{c.name}() given twice")
            seen[key] = c
        if "with_dtype" not in seen:
            raise DslError("a kernel needs .with_dtype(input=, acc=, output=): the grammar's constraint list makes it REQUIRED")
        if not self.is_conv and "with_layout" not in seen:
            raise DslError("a GEMM kernel needs .with_layout(A=, B=, C=): the grammar's constraint list makes it REQUIRED")
        d = seen["with_dtype"].kwargs
        for k in ("input", "acc", "output"):
            if k not in d:
                raise DslError(f".with_dtype() lacks {k}=")
            if d[k] not in _KNOWN_DTYPES:
                raise DslError(f".with_dtype({k}={d[k]}): not a DTYPE of the grammar")
        if d["acc"] not in ("fp32", "float32"):
            raise DslError(f".with_dtype(acc={d['acc']}): the matrix cores accumulate in fp32")
        if d["input"] not in _DTYPES or _DTYPES[d["input"]] == "f32":
            raise DslError(f".with_dtype(input={d['input']}): inputs are fp16, bf16, fp8_e4m3 or fp8_e5m2")
        if d["output"] not in _DTYPES or _ELEM_BYTES[_DTYPES[d["output"]]] == 1:
            raise DslError(f".with_dtype(output={d['output']}): outputs are fp16, bf16 or fp32")
        self.dt_in, self.dt_out = _DTYPES[d["input"]], _DTYPES[d["output"]]
        self.layouts = None
        if "with_layout" in seen:
            lay = seen["with_layout"].kwargs
            if self.is_conv:
                for k in ("input", "filter", "output"):
                    if lay.get(k) != "TensorNHWC":
                        raise DslError(f".with_layout({k}={lay.get(k)}): conv2d tensors are TensorNHWC (filter KRSC, output NPQK)")
            else:
                for k in ("A", "B", "C"):
                    if lay.get(k) not in ("RowMajor", "ColumnMajor"):
                        raise DslError(f".with_layout({k}={lay.get(k)}): RowMajor or ColumnMajor")
                if lay["C"] != "RowMajor":
                    raise DslError(".with_layout(C=ColumnMajor): the output is written row-major; swap the operands' roles, (A.B)^T = B^T.A^T")
                self.layouts = (lay["A"], lay["B"])
        t = dict(tile_m=0, tile_n=0, tile_k=0, stages=0, raster=0, iterator=0, split_k="none", slices=0, scheduler="default")
        if "with_tile" in seen:
            c = seen["with_tile"].kwargs
            t["tile_m"], t["tile_n"], t["tile_k"] = (self._int(c, k, "with_tile") for k in ("m", "n", "k"))
        if "with_stages" in seen:
            a = seen["with_stages"].args
            if len(a) != 1 or not isinstance(a[0], int) or a[0] < 1:
                raise DslError(".with_stages(n): one positive integer")
            t["stages"] = a[0]
        if ("with_tile" in seen) != ("with_stages" in seen):
            raise DslError("tile and stages name a kernel variant together: give both .with_tile (or .with_threadblockshape) and .with_stages, or neither")
        if "with_alignment" in seen:
            c = seen["with_alignment"].kwargs
            for k, dt in (("A", self.dt_in), ("B", self.dt_in), ("C", self.dt_out)):
                a = self._int(c, k, "with_alignment")
                if a < 1 or (a * _ELEM_BYTES[dt]) % 16:
                    raise DslError(f".with_alignment({k}={a}): (alignment * element_size) % 16 == 0 is required; {dt} elements are "
                                   f"{_ELEM_BYTES[dt]} bytes, so {k} >= {16 // _ELEM_BYTES[dt]} in steps of {16 // _ELEM_BYTES[dt]}")
        if "with_swizzle" in seen:
            pat = seen["with_swizzle"].kwargs.get("pattern")
            if pat == "StreamK":
                t["scheduler"] = "stream_k"
            elif pat in _SWIZZLE:
                t["raster"] = _SWIZZLE[pat]
            else:
                raise DslError(f".with_swizzle(pattern={pat}): Identity1, Identity2, Identity4, Identity8 or StreamK")
        if "with_iterator" in seen:
            a = seen["with_iterator"].args
            if not self.is_conv:
                raise DslError(".with_iterator() belongs to convolutions")
            if len(a) != 1 or a[0] not in ("analytic", "optimized", "fixed_channels", "few_channels", "fixed_stride_dilation"):
                raise DslError(f".with_iterator({a}): not an ITERATOR of the grammar")
            if a[0] not in _ITERATORS:
                raise DslError(f".with_iterator({a[0]}): not built; analytic (per-tap gather), optimized (the table's choice) and fixed_stride_dilation (resident patch) are")
            t["iterator"] = _ITERATORS[a[0]]
        if "with_split_k" in seen:
            c = seen["with_split_k"].kwargs
            if c.get("mode") not in ("none", "serial", "parallel"):
                raise DslError(f".with_split_k(mode={c.get('mode')}): none, serial or parallel")
            t["split_k"], t["slices"] = c["mode"], self._int(c, "slices", "with_split_k")
        if "with_scheduler" in seen:
            c = seen["with_scheduler"].kwargs
            tile = c.get("tile", "default")
            if tile not in ("default", "persistent", "stream_k", "streamk"):
                raise DslError(f".with_scheduler(tile={tile}): default, persistent or stream_k")
            if tile != "default":
                t["scheduler"] = "stream_k" if tile in ("stream_k", "streamk") else "persistent"
            if "splits" in c:
                if t["split_k"] != "none":
                    raise DslError(".with_scheduler(splits=) and .with_split_k() both name a K split")
                t["split_k"], t["slices"] = "parallel", self._int(c, "splits", "with_scheduler")
            for k in ("kernel", "epilogue"):
                if k in c:
                    self.ignored.append(f"with_scheduler({k}={c[k]})")
        self.scaling = None
        if "with_scaling" in seen:
            c = seen["with_scaling"].kwargs
            self.scaling = (float(c.get("alpha", 1.0)), float(c.get("beta", 0.0)))
        for n_, c in seen.items():
            if n_ in _NVIDIA_ONLY:
                self.ignored.append(repr(c))
            elif n_ not in ("with_dtype", "with_layout", "with_tile", "with_stages", "with_alignment", "with_swizzle",
                            "with_iterator", "with_split_k", "with_scheduler", "with_scaling"):
                raise DslError(f".{c.name}(): not a configuration of the grammar")
        self.tuning = t
        self._lower_chain()

    @staticmethod
    def _int(kw, key, where):
        v = kw.get(key)
        if not isinstance(v, int):
            raise DslError(f"{where}: {key}= must be an integer, got {v!r}")
        return v

    # -- epilogue chain -------------------------------------------------------------------------
    def _lower_chain(self):
        """steps: ("name", p0[, p1]) or ("name", operand) with operand the key launch() looks up."""
        steps = []
        if self.scaling:
            alpha, beta = self.scaling
            if alpha != 1.0:
                steps.append(("scale", alpha))
            if beta != 0.0:
                steps.append(("aux_load", "C", beta))        # D = alpha * acc + beta * C
        for c in self.chain_calls:
            n, a, kw = c.name, c.args, c.kwargs
            if n in _SIMPLE_ACT:
                steps.append((_SIMPLE_ACT[n],))
            elif n == "gelu":
                steps.append(("gelu_tanh" if self.gelu == "tanh" else "gelu_erf",))
            elif n == "leaky_relu":
                steps.append(("leaky_relu", float(kw["alpha"])) if "alpha" in kw else self._bad(c, "alpha= is required"))
            elif n == "elu":
                steps.append(("elu", float(kw.get("alpha", 1.0))))
            elif n in ("clip", "clamp"):
                if "min" not in kw or "max" not in kw:
                    self._bad(c, "min= and max= are required")
                steps.append(("clamp", float(kw["min"]), float(kw["max"])))
            elif n == "scale":
                steps.append(("scale", float(kw["alpha"])) if "alpha" in kw else self._bad(c, "alpha= is required"))
            elif n == "bias":
                steps.append(("bias", "bias"))
            elif n in ("per_channel_scale", "per_col_scale"):
                steps.append(("per_col_scale", "per_col_scale"))
            elif n == "per_row_scale":
                steps.append(("per_row_scale", "per_row_scale"))
            elif n in ("row_broadcast", "column_broadcast", "aux_load", "aux_store"):
                if len(a) != 1 or not isinstance(a[0], str):
                    self._bad(c, "one tensor identifier is required")
                steps.append((n, a[0]))
            elif n == "custom":
                self._bad(c, "custom expressions need a run-time compiler, which this library does not have")
            else:
                self._bad(c, "not an epilogue_op of the grammar")
        if len(steps) > ucl.MAX_EPI_STEPS:
            raise DslError(f"the chain lowers to {len(steps)} steps; the library's chain holds {ucl.MAX_EPI_STEPS}")
        self.steps = steps

    @staticmethod
    def _bad(call, why):
        raise DslError(f">> {call!r}: {why}")

    def operands(self):
        """Names of the tensor operands launch() expects in `tensors`, in chain order."""
        return [s[1] for s in self.steps if s[0] in ucl.Epilogue.TENSOR]

    # -- marshalling ----------------------------------------------------------------------------
    def make_tuning(self, workspace=0, workspace_bytes=0):
        return ucl.Tuning(workspace=workspace, workspace_bytes=workspace_bytes, **self.tuning)

    def make_epilogue(self, tensors, N, batch_rows=0):
        """tensors: name -> (device address, dtype) or (address, dtype, ld); matrices default to ld = N."""
        out = []
        for s in self.steps:
            if s[0] in ucl.Epilogue.TENSOR:
                if s[1] not in tensors:
                    raise DslError(f"epilogue operand {s[1]!r} of {s[0]}() was not passed to launch()")
                t = tensors[s[1]]
                is_mat = s[0] in ("aux_load", "aux_store")
                ld = t[2] if len(t) > 2 else (N if is_mat else 0)
                out.append((s[0], t[0], t[1], ld, batch_rows * N if is_mat else 0, s[2] if len(s) > 2 else 1.0))
            else:
                out.append(s)
        return ucl.Epilogue(out)

    def launch(self, A=None, B=None, D=None, tensors=None, stream=0, workspace=0, workspace_bytes=0, **shape):
        """Call the library.  gemm: M, N, K;  batched_gemm: batch, M, N, K;  grouped_gemm: M_g (host list), N, K
        and A / B / D the device addresses of the per-group pointer tables;  convolutions: N, H, W, C, Kout and
        optionally pad=(h, w), stride=, dil= (A = first operand, B = second, D = result, in the order of the
        C declaration).  Operands are packed in the layouts the program names."""
        tensors = tensors or {}
        tune = self.make_tuning(workspace, workspace_bytes)
        if self.is_conv:
            n, h, w, c, ko = (shape[k] for k in ("N", "H", "W", "C", "Kout"))
            r, s_ = self.filter
            pad, stride, dil = shape.get("pad", (0, 0)), shape.get("stride", (1, 1)), shape.get("dil", (1, 1))
            p = (h + 2 * pad[0] - dil[0] * (r - 1) - 1) // stride[0] + 1
            q = (w + 2 * pad[1] - dil[1] * (s_ - 1) - 1) // stride[1] + 1
            cols = {"conv2d_fprop": ko, "conv2d_dgrad": c, "conv2d_wgrad": r * s_ * c}[self.op]
            epi = self.make_epilogue(tensors, cols)
            fn = getattr(ucl, "ucl_" + self.op)
            return fn(n, h, w, c, ko, r, s_, pad[0], pad[1], stride[0], stride[1], dil[0], dil[1], A, self.dt_in, B,
                      self.dt_in, D, self.dt_out, epi, tune, stream)
        N, K = shape["N"], shape["K"]
        la, lb = self.layouts
        if self.op == "grouped_gemm":
            M_g = list(shape["M_g"])
            if self.expert_count != len(M_g):
                raise DslError(f"grouped_gemm(expert_count={self.expert_count}) launched with {len(M_g)} groups")
            if la != "RowMajor":
                raise DslError("grouped_gemm is built for A=RowMajor")
            b = (N, 1) if lb == "RowMajor" else (1, K)
            return ucl.ucl_grouped_gemm(M_g, N, K, A, self.dt_in, K, 1, B, self.dt_in, b[0], b[1], D, self.dt_out, N, 1,
                                        self.make_epilogue(tensors, N), tune, stream)
        M = shape["M"]
        a = (K, 1) if la == "RowMajor" else (1, M)
        b = (N, 1) if lb == "RowMajor" else (1, K)
        if self.op == "batched_gemm":
            return ucl.ucl_batched_gemm(shape["batch"], M, N, K, A, self.dt_in, a[0], a[1], M * K, B, self.dt_in, b[0], b[1],
                                        N * K, D, self.dt_out, N, 1, M * N, self.make_epilogue(tensors, N, batch_rows=M), tune, stream)
        return ucl.ucl_gemm(M, N, K, A, self.dt_in, a[0], a[1], B, self.dt_in, b[0], b[1], D, self.dt_out, N, 1,
                            self.make_epilogue(tensors, N), tune, stream)

    def __repr__(self):
        return f"Kernel({self.op}, {self.dt_in}->{self.dt_out}, tuning={self.tuning}, steps={self.steps})"


class Transpose:
    """Transform stage transpose(tensor, L1, L2 [, dtype_in, dtype_out])."""

    _PAIRS = {("NCL", "NLC"), ("NLC", "NCL"), ("NCHW", "NHWC"), ("NHWC", "NCHW")}

    def __init__(self, call):
        a = call.args
        if len(a) not in (3, 5) or call.kwargs:
            raise DslError(f"{call!r}: transpose(tensor, layout, layout [, dtype, dtype])")
        if a[0] not in ("input", "output", "weight"):
            raise DslError(f"{call!r}: the tensor is input, output or weight")
        if (a[1], a[2]) not in self._PAIRS:
            raise DslError(f"{call!r}: layouts NCL <-> NLC or NCHW <-> NHWC")
        self.tensor, self.src_layout, self.dst_layout = a[0], a[1], a[2]
        self.dt_src = self.dt_dst = None
        if len(a) == 5:
            for v in a[3:]:
                if v not in _DTYPES or _ELEM_BYTES[_DTYPES[v]] == 1:
                    raise DslError(f"{call!r}: the transform stage converts between fp32, fp16 and bf16")
            self.dt_src, self.dt_dst = _DTYPES[a[3]], _DTYPES[a[4]]

    def extents(self, channels, length):
        """(rows, cols) of the matrices the library transposes: channels-first sources have rows = C."""
        return (channels, length) if self.src_layout in ("NCL", "NCHW") else (length, channels)

    def launch(self, batch, channels, length, src, dst, dtype=None, stream=0):
        """length = L, or H * W for the 4-D layouts.  dtype: element type when the stage names none."""
        dt_src, dt_dst = self.dt_src or dtype, self.dt_dst or dtype
        if dt_src is None:
            raise DslError("this transpose stage names no element types: pass dtype=")
        rows, cols = self.extents(channels, length)
        return ucl.ucl_transpose(batch, rows, cols, src, dt_src, dst, dt_dst, stream)

    def __repr__(self):
        return f"Transpose({self.tensor}, {self.src_layout}->{self.dst_layout}, {self.dt_src}->{self.dt_dst})"


class Pipeline:
    """pipeline(stage, stage, ...): stages with explicit kernel boundaries, launched one after the
    other on one stream by the caller (each stage's launch())."""

    def __init__(self, stages):
        if not any(isinstance(s, Kernel) for s in stages):
            raise DslError("a pipeline needs at least one kernel stage")
        self.stages = stages

    def __repr__(self):
        return "Pipeline(" + ", ".join(repr(s) for s in self.stages) + ")"


def parse(text, gelu="erf"):
    """Parse a DSL program; returns a Kernel or a Pipeline.  gelu: "erf" (default) or "tanh"."""
    prog = _Parser(text).program()
    if gelu != "erf":
        for k in (prog.stages if isinstance(prog, Pipeline) else [prog]):
            if isinstance(k, Kernel):
                k.gelu = gelu
                k._lower_chain()
    return prog
