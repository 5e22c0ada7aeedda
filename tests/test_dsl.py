"""The DSL-text translator (host only): the paper's Sec. 3 example program and the grammar's own
template programs parse and lower to the expected library arguments; malformed or unsupported
programs are rejected with a reason.  The last test runs the example program on the GPU."""
import numpy as np
import pytest

from paper_2603_29010_amd import dsl, synth
from paper_2603_29010_amd.dsl import DslError

# Fig. "compilation pipeline", input box (Sec. 3): a GEMM with a fused bias -> GELU -> clip epilogue
PAPER_EXAMPLE = """
gemm()
  .with_dtype(input=fp16, acc=fp32, output=fp16)
  .with_layout(A=RowMajor, B=RowMajor, C=RowMajor)
  .with_arch(sm_90a)
  .with_threadblockshape(m=128, n=128, k=64)
  .with_stages(2)
  .with_alignment(A=8, B=8, C=8)
  .with_scheduler(kernel=tma, epilogue=tma)
  >> bias() >> gelu() >> clip(min=0, max=6)
"""


def test_paper_example_program_lowers_to_the_expected_call():
    k = dsl.parse(PAPER_EXAMPLE)
    assert isinstance(k, dsl.Kernel) and k.op == "gemm"
    assert (k.dt_in, k.dt_out) == ("f16", "f16") and k.layouts == ("RowMajor", "RowMajor")
    assert (k.tuning["tile_m"], k.tuning["tile_n"], k.tuning["tile_k"], k.tuning["stages"]) == (128, 128, 64, 2)
    assert k.steps == [("bias", "bias"), ("gelu_erf",), ("clamp", 0.0, 6.0)]
    assert k.operands() == ["bias"]
    # the NVIDIA-specific settings are accepted and have no effect
    assert any("sm_90a" in s for s in k.ignored) and "with_scheduler(kernel=tma)" in k.ignored
    assert dsl.parse(PAPER_EXAMPLE, gelu="tanh").steps[1] == ("gelu_tanh",)
    t = k.make_tuning().as_dict()
    assert (t["tile_m"], t["tile_k"], t["stages"]) == (128, 64, 2)


def test_grammar_template_programs():
    # the two template programs printed with the grammar's constraint list
    k = dsl.parse("""gemm().with_dtype(input=fp16, acc=fp32, output=fp16)
        .with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor).with_arch(sm_90a)
        .with_threadblockshape(m=256, n=128, k=64).with_alignment(A=8, B=8, C=8).with_stages(2)
        .with_scheduler(kernel=tma_cooperative, epilogue=tma_cooperative)""")
    assert k.layouts == ("RowMajor", "ColumnMajor") and k.steps == []
    with pytest.raises(DslError, match="inputs are fp16, bf16"):
        dsl.parse("""gemm().with_dtype(input=fp32, acc=fp32, output=fp32)
            .with_layout(A=RowMajor, B=RowMajor, C=RowMajor).with_arch(sm_90a)
            .with_threadblockshape(m=128, n=128, k=32).with_cluster(m=4, n=2, k=1)
            .with_alignment(A=4, B=4, C=4).with_stages(3).with_operand_swap(true)""")


def test_every_operation_knob_and_epilogue_op():
    k = dsl.parse("""conv2d_fprop(kernel_h=3, kernel_w=3)
        .with_dtype(input=bf16, acc=fp32, output=bf16)
        .with_layout(input=TensorNHWC, filter=TensorNHWC, output=TensorNHWC)
        .with_tile(m=256, n=128, k=32).with_stages(4).with_iterator(fixed_stride_dilation).with_swizzle(pattern=Identity4)
        >> bias() >> aux_load(residual) >> relu()""")
    assert k.op == "conv2d_fprop" and k.filter == (3, 3) and k.tuning["iterator"] == 2 and k.tuning["raster"] == 4
    assert k.steps == [("bias", "bias"), ("aux_load", "residual"), ("relu",)] and k.operands() == ["bias", "residual"]
    k = dsl.parse("conv1d_fprop(kernel_w=5).with_dtype(input=fp16, acc=fp32, output=fp32)")
    assert k.op == "conv2d_fprop" and k.filter == (1, 5)
    k = dsl.parse("""conv2d_wgrad(kernel_h=3, kernel_w=3).with_dtype(input=bf16, acc=fp32, output=fp32)
        .with_split_k(mode=serial, slices=16)""")
    assert k.op == "conv2d_wgrad" and (k.tuning["split_k"], k.tuning["slices"]) == ("serial", 16)
    k = dsl.parse("""grouped_gemm(expert_count=16).with_dtype(input=bf16, acc=fp32, output=bf16)
        .with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor) >> silu()""")
    assert k.expert_count == 16 and k.steps == [("silu",)]
    k = dsl.parse("""batched_gemm().with_dtype(input=e4m3, acc=float32, output=bfloat16)
        .with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor).with_scaling(alpha=0.5, beta=2)
        .with_scheduler(tile=persistent, splits=4)
        >> per_row_scale() >> per_channel_scale() >> row_broadcast(rb) >> column_broadcast(cb) >> mish() >> sigmoid()""")
    assert k.dt_in == "e4m3" and k.tuning["scheduler"] == "persistent" and (k.tuning["split_k"], k.tuning["slices"]) == ("parallel", 4)
    assert k.steps[:2] == [("scale", 0.5), ("aux_load", "C", 2.0)] and len(k.steps) == 8
    assert k.operands() == ["C", "per_row_scale", "per_col_scale", "rb", "cb"]
    with pytest.raises(DslError, match="chain holds 8"):
        dsl.parse("""gemm().with_dtype(input=bf16, acc=fp32, output=fp32).with_layout(A=RowMajor, B=RowMajor, C=RowMajor)
            >> relu() >> tanh() >> hardswish() >> mish() >> silu() >> gelu() >> sigmoid() >> relu() >> tanh()""")
    k = dsl.parse("""gemm().with_dtype(input=bf16, acc=fp32, output=fp32).with_layout(A=ColumnMajor, B=RowMajor, C=RowMajor)
        >> leaky_relu(alpha=0.1) >> elu() >> elu(alpha=1.5) >> clamp(min=-1, max=1.5) >> scale(alpha=-2.5) >> aux_store(saved)""")
    assert k.steps == [("leaky_relu", 0.1), ("elu", 1.0), ("elu", 1.5), ("clamp", -1.0, 1.5), ("scale", -2.5), ("aux_store", "saved")]


def test_pipeline_with_transform_stages():
    p = dsl.parse("""pipeline(
        transpose(input, NCHW, NHWC, fp32, bf16),
        conv2d_fprop(kernel_h=3, kernel_w=3).with_dtype(input=bf16, acc=fp32, output=bf16) >> bias() >> relu(),
        transpose(output, NHWC, NCHW, bf16, fp32))""")
    assert isinstance(p, dsl.Pipeline) and len(p.stages) == 3
    t0, k, t2 = p.stages
    assert (t0.src_layout, t0.dst_layout, t0.dt_src, t0.dt_dst) == ("NCHW", "NHWC", "f32", "bf16")
    assert t0.extents(64, 56 * 56) == (64, 3136) and t2.extents(128, 56 * 56) == (3136, 128)
    assert k.op == "conv2d_fprop" and t2.tensor == "output"
    t = dsl.parse("pipeline(transpose(input, NCL, NLC), gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor))")
    assert t.stages[0].dt_src is None


@pytest.mark.parametrize("text,why", [
    ("gemm().with_layout(A=RowMajor, B=RowMajor, C=RowMajor)", "REQUIRED"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16)", "REQUIRED"),
    ("gemm().with_dtype(input=fp16, acc=fp16, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor)", "accumulate in fp32"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=ColumnMajor)", "swap the operands"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor).with_alignment(A=4, B=8, C=8)", r"% 16 == 0"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor).with_tile(m=128, n=128, k=64)", "together"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor) >> custom('x*2')", "run-time compiler"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor) >> relu() .with_stages(2)", "before the first >>"),
    ("gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor) >> softmax()", "not an epilogue_op"),
    ("conv3d_fprop(kernel_d=3, kernel_h=3, kernel_w=3).with_dtype(input=fp16, acc=fp32, output=fp16)", "builds gemm"),
    ("conv2d_fprop(kernel_h=3, kernel_w=3).with_dtype(input=fp16, acc=fp32, output=fp16).with_iterator(few_channels)", "not built"),
    ("gemm().with_dtype(input=int8, acc=int32, output=int8).with_layout(A=RowMajor, B=RowMajor, C=RowMajor)", "accumulate in fp32"),
    ("gemm(.with_dtype(input=fp16, acc=fp32, output=fp16)", "expected"),
    ("matmul().with_dtype(input=fp16, acc=fp32, output=fp16)", "unknown operation"),
    ("pipeline(transpose(input, NCL, NLC))", "at least one kernel stage"),
    ("pipeline(transpose(input, NCL, NHWC), gemm().with_dtype(input=fp16, acc=fp32, output=fp16).with_layout(A=RowMajor, B=RowMajor, C=RowMajor))", "layouts"),
])
def test_rejected_programs_say_why(text, why):
    with pytest.raises(DslError, match=why):
        dsl.parse(text)


@pytest.mark.gpu
def test_paper_example_program_runs_and_matches_the_oracle():
    import torch
    import oracle
    import parity
    from paper_2603_29010_amd.workload import DeviceWorkload
    k = dsl.parse(PAPER_EXAMPLE)
    spec = synth.gemm_spec(264, 392, 200, dt_in="f16", dt_out="f16", a_layout="row", b_layout="row", scale=0.5,
                           epilogue=("bias", "gelu_erf", ("clamp", 0.0, 6.0)))
    w = DeviceWorkload(spec)                       # device buffers only; the launch goes through the translator
    (bias_key,) = spec["tensors"]
    bias = [t for t in w.keep if t.numel() == spec["N"]][0]
    k.launch(M=spec["M"], N=spec["N"], K=spec["K"], A=w.A.data_ptr(), B=w.B.data_ptr(), D=w.D.data_ptr(),
             tensors={"bias": (bias.data_ptr(), "f16")}, stream=torch.cuda.current_stream().cuda_stream)
    ref, absacc = parity.oracle_result(spec)
    parity.compare(w.result(), ref, absacc, spec, "paper example through the translator")
    assert w.result().max() <= 6.0 and w.result().min() >= 0.0


@pytest.mark.gpu
def test_scheduler_split_k_and_fp8_programs_run_through_the_translator():
    import torch
    import parity
    import paper_2603_29010_amd as ucl
    from paper_2603_29010_amd.workload import DeviceWorkload
    st = torch.cuda.current_stream().cuda_stream
    # the persistent tile scheduler, tile named in the program
    k = dsl.parse("""gemm().with_dtype(input=bf16, acc=fp32, output=fp32).with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor)
        .with_tile(m=128, n=128, k=32).with_stages(4).with_scheduler(tile=persistent)""")
    spec = synth.gemm_spec(1100, 1300, 136, dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    k.launch(M=1100, N=1300, K=136, A=w.A.data_ptr(), B=w.B.data_ptr(), D=w.D.data_ptr(), stream=st)
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
    # split-K in parallel mode with a caller workspace: more than two slices, i.e. the reduction kernel between the launches
    k = dsl.parse("""gemm().with_dtype(input=bf16, acc=fp32, output=fp32).with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor)
        .with_split_k(mode=parallel, slices=6)""")
    spec = synth.gemm_spec(200, 136, 1992, dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), st)
    k.launch(M=200, N=136, K=1992, A=w.A.data_ptr(), B=w.B.data_ptr(), D=w.D.data_ptr(), stream=st,
             workspace=ws.data_ptr(), workspace_bytes=ws.numel())
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
    # the data gradient of a 3x3 convolution through the resident-patch iterator (128 output channels)
    k = dsl.parse("""conv2d_dgrad(kernel_h=3, kernel_w=3).with_dtype(input=bf16, acc=fp32, output=fp32)
        .with_iterator(fixed_stride_dilation)""")
    spec = synth.conv_grad_spec("dgrad", Nb=2, H=13, W=11, C=24, Ko=128, R=3, S=3, pad=(1, 1), dt_out="f32", integer=True)
    w = DeviceWorkload(spec)
    k.launch(N=2, H=13, W=11, C=24, Kout=128, pad=(1, 1), A=w.A.data_ptr(), B=w.B.data_ptr(), D=w.D.data_ptr(), stream=st)
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
    # grouped GEMM on fp8 inputs
    k = dsl.parse("""grouped_gemm(expert_count=4).with_dtype(input=fp8_e4m3, acc=fp32, output=fp32)
        .with_layout(A=RowMajor, B=ColumnMajor, C=RowMajor)""")
    spec = synth.grouped_spec([130, 0, 64, 300], 136, 208, dt_in="e4m3", dt_out="f32", epilogue=(), integer=True)
    w = DeviceWorkload(spec)
    k.launch(M_g=spec["M_g"], N=136, K=208, A=w.tabA.data_ptr(), B=w.tabB.data_ptr(), D=w.tabD.data_ptr(), stream=st)
    assert np.array_equal(w.result(), parity.orc_run.run(spec))
