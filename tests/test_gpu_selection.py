"""The selection table against measurement: on a handful of problem shapes every built variant that
serves the problem is timed, and the table's pick must not be slower than the fastest of them by
more than 10 % (the table aims at 6 %; launch-to-launch noise on a shared box is a few percent)."""
import statistics

import pytest
import torch

import paper_2603_29010_amd as ucl
from paper_2603_29010_amd import synth
from paper_2603_29010_amd.binding import Tuning
from paper_2603_29010_amd.workload import DeviceWorkload

from test_gpu_parity import built

pytestmark = pytest.mark.gpu


def time_us(w, tune, launches=20, replays=5):
    for _ in range(5):
        w.run(tune=tune)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(launches):
            w.run(tune=tune)
    g.replay()
    torch.cuda.synchronize()
    out = []
    for _ in range(replays):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        g.replay()
        b.record()
        torch.cuda.synchronize()
        out.append(a.elapsed_time(b) * 1e3 / launches)
    return statistics.median(out)


def spin_up(w):
    for _ in range(300):
        w.run()
    torch.cuda.synchronize()


SHAPES = {
    "gemm 4096^3": lambda: synth.config(2),
    "gemm 2048^3": lambda: synth.gemm_spec(2048, 2048, 2048, scale=1 / 45, epilogue=("bias", "gelu_tanh")),
    "gemm 1024x1024x8192": lambda: synth.gemm_spec(1024, 1024, 8192, scale=1 / 90, epilogue=("bias", "relu")),
    "gemm 8192x512x512": lambda: synth.gemm_spec(8192, 512, 512, scale=1 / 22, epilogue=("silu",)),
    "gemm 256^3": lambda: synth.gemm_spec(256, 256, 256, epilogue=("bias", "relu")),
    "batched 64x512x512x128 fp16 -> fp32": lambda: synth.config(3),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_table_pick_is_near_the_fastest_built_variant(name):
    spec = SHAPES[name]()
    w = DeviceWorkload(spec, poison=False)
    spin_up(w)
    pick = w.selected()
    pick_key = (pick["tile_m"], pick["tile_n"], pick["tile_k"], pick["stages"])
    times = {}
    for tile in built(0, f16=int(spec["dt_in"] == "f16")):
        times[tile] = time_us(w, Tuning(*tile))
    assert pick_key in times, (pick_key, sorted(times))
    t_pick = min(times[pick_key], time_us(w, None))
    best = min(times, key=times.get)
    if t_pick > 1.10 * times[best]:
        # one more reading of the two before judging (a neighbour's burst on a shared box moves a 20-launch reading by more)
        t_pick = min(t_pick, time_us(w, None), time_us(w, Tuning(*pick_key)))
        times[best] = max(times[best], time_us(w, Tuning(*best)))
    assert t_pick <= 1.10 * times[best], (f"{name}: the table picks {pick_key} at {t_pick:.1f} us, "
                                          f"{best} runs {times[best]:.1f} us; all: " +
                                          ", ".join(f"{k}: {v:.1f}" for k, v in sorted(times.items(), key=lambda kv: kv[1])))


SPLIT_SHAPES = {
    "gemm 256x256x16384": (lambda: synth.gemm_spec(256, 256, 16384, dist="uniform", scale=0.05, epilogue=("bias", "relu")), 0, None),
    "gemm 512x512x8192 -> fp32": (lambda: synth.gemm_spec(512, 512, 8192, dt_out="f32", epilogue=()), 0, None),
    "wgrad 32x56x56, 64 -> 128 channels, 3x3": (lambda: synth.conv_grad_spec("wgrad", dt_out="f32", Nb=32, H=56, W=56, C=64, Ko=128, R=3, S=3,
                                                                               pad=(1, 1)), 4, 5),
}


@pytest.mark.parametrize("mode", ["parallel", "serial"])
@pytest.mark.parametrize("name", list(SPLIT_SHAPES))
def test_split_k_pick_is_near_the_fastest_built_variant(name, mode):
    # with split-K asked for and no tile named, the choice follows a model of its own (operand copy traffic, the
    # workgroups' copy chains, the partial tiles' trip through memory): within 15 % of the best tile, slices left to the library
    make, op_mode, la = SPLIT_SHAPES[name]
    w = DeviceWorkload(make(), poison=False)
    ws = torch.empty(128 << 20, dtype=torch.uint8, device="cuda")
    ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    tune = lambda *tile: Tuning(*tile, split_k=mode, workspace=ws.data_ptr(), workspace_bytes=ws.numel())
    for _ in range(100):
        w.run(tune=tune())
    torch.cuda.synchronize()
    times = {tile: time_us(w, tune(*tile)) for tile in (built(op_mode, la=la, lb=4) if op_mode == 4 else built(0))}
    t_pick = time_us(w, tune())
    best = min(times, key=times.get)
    if t_pick > 1.15 * times[best]:
        t_pick = min(t_pick, time_us(w, tune()))
        times[best] = max(times[best], time_us(w, tune(*best)))
    assert t_pick <= 1.15 * times[best], (f"{name} ({mode}): the library's choice runs {t_pick:.1f} us, {best} runs {times[best]:.1f} us; all: " +
                                          ", ".join(f"{k}: {v:.1f}" for k, v in sorted(times.items(), key=lambda kv: kv[1])))


CONV_SHAPES = {
    "fprop 32x56x56, 64 -> 128": (lambda: synth.config(5), 2),
    "fprop 32x28x28, 128 -> 128": (lambda: synth.conv_spec(Nb=32, H=28, W=28, C=128, Ko=128, R=3, S=3), 2),
    "dgrad 32x56x56, 64 <- 128": (lambda: synth.conv_grad_spec("dgrad", Nb=32, H=56, W=56, C=64, Ko=128, R=3, S=3, pad=(1, 1)), 3),
    "dgrad 32x56x56, 64 <- 64": (lambda: synth.conv_grad_spec("dgrad", Nb=32, H=56, W=56, C=64, Ko=64, R=3, S=3, pad=(1, 1)), 3),
}


@pytest.mark.parametrize("name", list(CONV_SHAPES))
def test_conv_pick_is_near_the_fastest_built_variant(name):
    # 3x3 convolutions that the resident-patch kernels serve: the table chooses between them and the per-tap gather kernels
    make, mode = CONV_SHAPES[name]
    spec = make()
    w = DeviceWorkload(spec, poison=False)
    spin_up(w)
    channels = spec["C"] if mode == 2 else spec["Ko"]
    lb = 0 if mode == 2 else 4
    times = {}
    for tile in built(mode, la=2, lb=lb):
        times[tile + ("gather",)] = time_us(w, Tuning(*tile, iterator=1))
    for tile in built(mode, la=3, lb=lb, patch_c=channels):
        times[tile + ("patch",)] = time_us(w, Tuning(*tile, iterator=2))
    t_pick = time_us(w, None)
    best = min(times, key=times.get)
    if t_pick > 1.15 * times[best]:
        t_pick = min(t_pick, time_us(w, None))
        times[best] = max(times[best], time_us(w, Tuning(*best[:4], iterator=1 if best[4] == "gather" else 2)))
    assert t_pick <= 1.15 * times[best], (f"{name}: the table's choice {w.selected()} runs {t_pick:.1f} us, {best} runs {times[best]:.1f} us; all: " +
                                          ", ".join(f"{k}: {v:.1f}" for k, v in sorted(times.items(), key=lambda kv: kv[1])))
