"""Seeded random shapes, layouts, types and chains through the table's own kernel choice, against the oracle."""
import numpy as np
import pytest

from paper_2603_29010_amd import synth

import parity

pytestmark = pytest.mark.gpu

CHAINS = [(), ("bias", "relu"), ("bias", "gelu_tanh"), ("silu",), (("scale", 0.5), "bias", "aux_load", "relu"),
          ("aux_load",), ("per_row_scale", "bias", "sigmoid")]


def _dims(rng, lo, hi, mult):
    return int(rng.integers(lo // mult, hi // mult + 1)) * mult


@pytest.mark.parametrize("seed", range(48))
def test_random_problem(seed):
    rng = np.random.default_rng(20260329 + seed)
    kind = ["gemm", "gemm", "batched", "grouped", "conv"][seed % 5]
    exact = bool(rng.integers(0, 2))
    dt_in = ["bf16", "f16"][int(rng.integers(0, 2))]
    dt_out = "f32" if exact else ["bf16", "f16", "f32"][int(rng.integers(0, 3))]
    chain = () if exact else CHAINS[int(rng.integers(0, len(CHAINS)))]
    if kind == "gemm":
        al, bl = ["row", "col"][int(rng.integers(0, 2))], ["col", "row"][int(rng.integers(0, 2))]
        M = _dims(rng, 8, 700, 8 if al == "col" else 1)
        N = _dims(rng, 8, 700, 8 if bl == "row" else 1)
        K = _dims(rng, 8, 520, 1 if (al == "col" and bl == "row") else 8)
        spec = synth.gemm_spec(M, N, K, dt_in=dt_in, dt_out=dt_out, a_layout=al, b_layout=bl, epilogue=chain,
                               integer=exact, seed=synth.BASE_SEED + 100 + seed)
        label = f"gemm {M}x{N}x{K} {al}/{bl} {dt_in}->{dt_out} {chain}"
    elif kind == "batched":
        b, M, N, K = int(rng.integers(1, 7)), _dims(rng, 8, 300, 1), _dims(rng, 8, 300, 1), _dims(rng, 8, 264, 8)
        chain = chain if "per_row_scale" not in chain else ("bias", "relu")
        spec = synth.batched_spec(b, M, N, K, dt_in=dt_in, dt_out=dt_out, epilogue=list(chain), integer=exact,
                                  seed=synth.BASE_SEED + 100 + seed)
        label = f"batched {b}x{M}x{N}x{K} {dt_in}->{dt_out} {chain}"
    elif kind == "grouped":
        G = int(rng.integers(1, 9))
        M_g = [int(rng.integers(0, 400)) for _ in range(G)]
        M_g[int(rng.integers(0, G))] = 0
        if sum(M_g) == 0:
            M_g[0] = 17
        bl = ["col", "row"][int(rng.integers(0, 2))]
        N, K = _dims(rng, 8, 400, 8), _dims(rng, 8, 264, 8)
        act = () if exact else [("silu",), ("relu",), ()][int(rng.integers(0, 3))]
        spec = synth.grouped_spec(M_g, N, K, dt_in=dt_in, dt_out=dt_out, epilogue=act, integer=exact, b_layout=bl,
                                  seed=synth.BASE_SEED + 100 + seed)
        label = f"grouped {M_g} N={N} K={K} B {bl} {dt_in}->{dt_out} {act}"
    else:
        patch = bool(rng.integers(0, 2))
        Nb, H, W = int(rng.integers(1, 5)), int(rng.integers(1, 20)), int(rng.integers(1, 20))
        if patch:
            C, R, S, pad, stride, dil = 64, 3, 3, (1, 1), (1, 1), (1, 1)
        else:
            C = _dims(rng, 8, 72, 8)
            R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
            pad = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
            stride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
            dil = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
            H, W = H + dil[0] * (R - 1), W + dil[1] * (S - 1)
        Ko = _dims(rng, 8, 200, 1)
        chain = chain if "per_row_scale" not in chain else ("bias", "aux_load", "relu")
        spec = synth.conv_spec(Nb, H, W, C, Ko, R, S, pad=pad, stride=stride, dil=dil, dt_in=dt_in, dt_out=dt_out,
                               epilogue=chain, integer=exact, seed=synth.BASE_SEED + 100 + seed)
        label = f"conv {Nb}x{H}x{W}x{C}->{Ko} {R}x{S} pad{pad} str{stride} dil{dil} {dt_in}->{dt_out} {chain}"
    if exact:
        parity.check_exact(spec, None, label=label)
    else:
        parity.check(spec, None, label=label)


_WS = {}


def _workspace():
    import torch
    import paper_2603_29010_amd as ucl
    ws = _WS.get("buf")
    if ws is None:
        ws = torch.empty(192 << 20, dtype=torch.uint8, device="cuda")
        ucl.ucl_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        _WS["buf"] = ws
    return ws


@pytest.mark.parametrize("seed", range(40))
def test_random_problem_under_a_random_schedule(seed):
    """The scheduling knobs on random GEMM shapes (kernel left to the library): split-K serial / parallel with a random
    slice count, the persistent and the stream-K scheduler, fp8 inputs; all on one workspace, whose counters every
    call must leave zero."""
    import torch
    from paper_2603_29010_amd.binding import Tuning, WORKSPACE_COUNTER_BYTES
    rng = np.random.default_rng(77001 + seed)
    ws = _workspace()
    knob = ["serial", "parallel", "persistent", "stream_k"][seed % 4]
    exact = bool(rng.integers(0, 2))
    fp8 = knob in ("serial", "parallel") and bool(rng.integers(0, 3) == 0)      # the schedulers are built for 16-bit inputs
    dt_in = ["e4m3", "e5m2"][int(rng.integers(0, 2))] if fp8 else ["bf16", "f16"][int(rng.integers(0, 2))]
    dt_out = "f32" if exact else ["bf16", "f32"][int(rng.integers(0, 2))]
    chain = () if exact else CHAINS[int(rng.integers(0, len(CHAINS)))]
    kmult = 16 if fp8 else 8
    batched = bool(rng.integers(0, 4) == 0)
    M, N = _dims(rng, 8, 900, 1), _dims(rng, 8, 900, 1)
    K = _dims(rng, 64, 3000 if knob != "persistent" else 400, kmult)
    if batched:
        b = int(rng.integers(2, 5))
        chain = chain if "per_row_scale" not in chain else ("bias", "relu")
        spec = synth.batched_spec(b, M // 2 + 8, N // 2 + 8, K, dt_in=dt_in, dt_out=dt_out, epilogue=list(chain), integer=exact,
                                  seed=synth.BASE_SEED + 500 + seed)
    else:
        spec = synth.gemm_spec(M, N, K, dt_in=dt_in, dt_out=dt_out, epilogue=chain, integer=exact, seed=synth.BASE_SEED + 500 + seed)
    kw = dict(workspace=ws.data_ptr(), workspace_bytes=ws.numel())
    if knob in ("serial", "parallel"):
        tune = Tuning(split_k=knob, slices=int(rng.integers(0, 12)), **kw)
    elif knob == "persistent":
        tune = Tuning(scheduler="persistent")
    else:
        tune = Tuning(scheduler="stream_k", **kw)
    label = f"{'batched' if batched else 'gemm'} {M}x{N}x{K} {dt_in}->{dt_out} {chain} under {knob}"
    if exact:
        parity.check_exact(spec, tune, label=label)
    else:
        parity.check(spec, tune, label=label)
    torch.cuda.synchronize()
    assert int(ws[:WORKSPACE_COUNTER_BYTES].count_nonzero().item()) == 0, label
