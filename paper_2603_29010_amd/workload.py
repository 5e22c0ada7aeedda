"""Put a synthetic workload dict (see synth.py) on the GPU and run it through the C ABI.

PyTorch is used for device memory and streams only: tensors are raw storage (int16 for
bf16 / fp16 bit patterns), every arithmetic step runs inside libucl.so.
"""
import numpy as np
import torch

from . import binding as ucl
from . import synth

_RAW = {"bf16": np.int16, "f16": np.int16, "f32": np.float32, "e4m3": np.uint8, "e5m2": np.uint8}
_TENSOR_OPS = ucl.Epilogue.TENSOR


def _to_device(arr, dtype, device):
    raw = np.ascontiguousarray(arr).view(_RAW[dtype])
    return torch.from_numpy(raw).to(device)


class DeviceWorkload:
    """Device-resident operands + output of one workload; `run()` enqueues exactly one ucl_* call."""

    def __init__(self, spec, device="cuda:0", poison=True):
        self.spec = spec
        self.device = torch.device(device)
        self.op = spec["op"]
        dt_in, dt_out = spec["dt_in"], spec["dt_out"]
        self.keep = []
        if self.op == "conv2d_fprop":
            self.A = _to_device(spec["x"], dt_in, self.device)
            self.B = _to_device(spec["w"], dt_in, self.device)
            self.out_shape = (spec["M"], spec["N"])
        elif self.op in ("conv2d_dgrad", "conv2d_wgrad"):
            self.A = _to_device(spec["dy"], dt_in, self.device)
            self.B = _to_device(spec["w" if self.op == "conv2d_dgrad" else "x"], dt_in, self.device)
            self.out_shape = (spec["M"], spec["N"])
        else:
            self.A = _to_device(spec["A"], dt_in, self.device)
            self.B = _to_device(spec["B"], dt_in, self.device)
            if self.op == "gemm":
                self.out_shape = (spec["M"], spec["N"])
            elif self.op == "batched_gemm":
                self.out_shape = (spec["batch"], spec["M"], spec["N"])
            else:
                self.out_shape = (int(sum(spec["M_g"])), spec["N"])
        tdt = torch.float32 if dt_out == "f32" else torch.int16
        self.D = torch.empty(self.out_shape, dtype=tdt, device=self.device)
        if poison:
            # NaN pattern in every output format: an element the kernel fails to write is caught
            self.D.fill_(float("nan") if dt_out == "f32" else 0x7FC1)
        self.aux_out = {}
        self._build_epilogue()
        if self.op == "grouped_gemm":
            self._build_tables()

    # -- epilogue -------------------------------------------------------------------------------
    def _build_epilogue(self):
        spec = self.spec
        steps = []
        grouped = self.op == "grouped_gemm"
        N = spec["N"]
        for st in spec["epilogue"]:
            name = st[0]
            if name in _TENSOR_OPS:
                if name == "aux_store":
                    dt = st[2]
                    t = torch.zeros(self.out_shape, dtype=torch.float32 if dt == "f32" else torch.int16,
                                    device=self.device)
                    self.aux_out[st[1]] = (t, dt)
                else:
                    arr, dt = spec["tensors"][st[1]]
                    t = _to_device(arr, dt, self.device)
                self.keep.append(t)
                is_mat = name in ("aux_load", "aux_store")
                ld = N if is_mat else 0
                bs = spec["M"] * N if (is_mat and self.op == "batched_gemm") else 0
                p0 = float(st[2]) if (name == "aux_load" and len(st) > 2) else 1.0
                if grouped:
                    ptr = self._group_table(t, is_mat, name in ("per_row_scale", "column_broadcast"))
                else:
                    ptr = t.data_ptr()
                steps.append((name, ptr, dt, ld, bs, p0))
            else:
                steps.append(tuple(st))
        self.epi = ucl.Epilogue(steps)

    def _group_table(self, t, is_matrix, by_row):
        """Per-group pointers into a packed operand (matrices / row vectors) or a shared vector."""
        M_g = self.spec["M_g"]
        offs = np.concatenate([[0], np.cumsum(M_g)])[:-1]
        esz = t.element_size()
        if is_matrix:
            addr = [t.data_ptr() + int(o) * self.spec["N"] * esz for o in offs]
        elif by_row:
            addr = [t.data_ptr() + int(o) * esz for o in offs]
        else:
            # n-indexed vectors: row g of a [groups, N rounded up to 8] array
            addr = [t.data_ptr() + g * t.shape[-1] * esz for g in range(len(M_g))]
        tab = torch.tensor(addr, dtype=torch.int64, device=self.device)
        self.keep.append(tab)
        return tab.data_ptr()

    def _build_tables(self):
        spec = self.spec
        M_g = spec["M_g"]
        offs = np.concatenate([[0], np.cumsum(M_g)])[:-1]
        K, N = spec["K"], spec["N"]
        esz_in, esz_out = self.A.element_size(), self.D.element_size()
        a = [self.A.data_ptr() + int(o) * K * esz_in for o in offs]
        b = [self.B.data_ptr() + g * N * K * esz_in for g in range(len(M_g))]
        d = [self.D.data_ptr() + int(o) * N * esz_out for o in offs]
        self.tabA = torch.tensor(a, dtype=torch.int64, device=self.device)
        self.tabB = torch.tensor(b, dtype=torch.int64, device=self.device)
        self.tabD = torch.tensor(d, dtype=torch.int64, device=self.device)

    # -- launch ---------------------------------------------------------------------------------
    def run(self, tune=None, stream=None):
        s = self.spec
        st = stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream
        if self.op == "gemm":
            ucl.ucl_gemm(s["M"], s["N"], s["K"], self.A.data_ptr(), s["dt_in"], *s["a_strides"],
                         self.B.data_ptr(), s["dt_in"], *s["b_strides"], self.D.data_ptr(), s["dt_out"],
                         s["N"], 1, self.epi, tune, st)
        elif self.op == "batched_gemm":
            a, b = s["a_strides"], s["b_strides"]
            ucl.ucl_batched_gemm(s["batch"], s["M"], s["N"], s["K"], self.A.data_ptr(), s["dt_in"], a[0], a[1],
                                 a[2], self.B.data_ptr(), s["dt_in"], b[0], b[1], b[2], self.D.data_ptr(),
                                 s["dt_out"], s["N"], 1, s["M"] * s["N"], self.epi, tune, st)
        elif self.op == "grouped_gemm":
            ucl.ucl_grouped_gemm(s["M_g"], s["N"], s["K"], self.tabA.data_ptr(), s["dt_in"], *s["a_strides"],
                                 self.tabB.data_ptr(), s["dt_in"], *s["b_strides"], self.tabD.data_ptr(),
                                 s["dt_out"], s["N"], 1, self.epi, tune, st)
        elif self.op in ("conv2d_dgrad", "conv2d_wgrad"):
            fn = ucl.ucl_conv2d_dgrad if self.op == "conv2d_dgrad" else ucl.ucl_conv2d_wgrad
            fn(s["Nb"], s["H"], s["W"], s["C"], s["Ko"], s["R"], s["S"], s["pad"][0], s["pad"][1], s["stride"][0],
               s["stride"][1], s["dil"][0], s["dil"][1], self.A.data_ptr(), s["dt_in"], self.B.data_ptr(), s["dt_in"],
               self.D.data_ptr(), s["dt_out"], self.epi, tune, st)
        else:
            ucl.ucl_conv2d_fprop(s["Nb"], s["H"], s["W"], s["C"], s["Ko"], s["R"], s["S"], s["pad"][0],
                                 s["pad"][1], s["stride"][0], s["stride"][1], s["dil"][0], s["dil"][1],
                                 self.A.data_ptr(), s["dt_in"], self.B.data_ptr(), s["dt_in"],
                                 self.D.data_ptr(), s["dt_out"], self.epi, tune, st)

    # -- results --------------------------------------------------------------------------------
    def result_bits(self):
        torch.cuda.synchronize(self.device)
        a = self.D.cpu().numpy()
        return a if self.spec["dt_out"] == "f32" else a.view(np.uint16)

    def result(self):
        """Output as float64 values (exact decode of what the kernel stored)."""
        return synth.bits_to_f64(self.result_bits(), self.spec["dt_out"])

    def aux_result(self, key):
        torch.cuda.synchronize(self.device)
        t, dt = self.aux_out[key]
        a = t.cpu().numpy()
        return synth.bits_to_f64(a if dt == "f32" else a.view(np.uint16), dt)

    # -- bookkeeping for the benchmark ----------------------------------------------------------
    def _problem_kwargs(self):
        s = self.spec
        if self.op.startswith("conv2d"):
            return dict(conv=(s["Nb"], s["H"], s["W"], s["C"], s["Ko"], s["R"], s["S"], s["pad"][0], s["pad"][1],
                              s["stride"][0], s["stride"][1], s["dil"][0], s["dil"][1]))
        kw = dict(N=s["N"], K=s["K"], a_layout="k" if s["a_strides"][1] == 1 else "mn",
                  b_layout="k" if s["b_strides"][0] == 1 else "mn")
        if self.op == "grouped_gemm":
            kw["M_g"] = s["M_g"]
        else:
            kw["M"] = s["M"]
            if self.op == "batched_gemm":
                kw["batch"] = s["batch"]
        return kw

    def selected(self):
        """The kernel the selection table picks for this workload (what run(tune=None) launches)."""
        s = self.spec
        return ucl.ucl_select_tuning(self.op, s["dt_in"], s["dt_out"], **self._problem_kwargs())

    def sol(self, hw=None):
        s = self.spec
        if self.op == "gemm":
            return ucl.ucl_sol_bound("gemm", s["dt_in"], s["dt_out"], hw=hw, M=s["M"], N=s["N"], K=s["K"], epi=self.epi)
        if self.op == "batched_gemm":
            return ucl.ucl_sol_bound("batched_gemm", s["dt_in"], s["dt_out"], hw=hw, batch=s["batch"], M=s["M"],
                                     N=s["N"], K=s["K"], epi=self.epi)
        if self.op == "grouped_gemm":
            return ucl.ucl_sol_bound("grouped_gemm", s["dt_in"], s["dt_out"], hw=hw, M_g=s["M_g"], N=s["N"],
                                     K=s["K"], epi=self.epi)
        return ucl.ucl_sol_bound(self.op, s["dt_in"], s["dt_out"], hw=hw, epi=self.epi,
                                 conv=(s["Nb"], s["H"], s["W"], s["C"], s["Ko"], s["R"], s["S"], s["pad"][0],
                                       s["pad"][1], s["stride"][0], s["stride"][1], s["dil"][0], s["dil"][1]))
