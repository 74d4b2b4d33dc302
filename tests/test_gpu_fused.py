"""GPU parity of the fused layer path: permute-gather folded into the first GEMM's row loads and
the gate-weighted scatter-combine into the second GEMM's stores.  Checked against the oracle and,
bit for bit, against the path with separate gather / combine passes."""
import numpy as np
import pytest
import torch

from gpu_util import assert_close, layer_inputs, make_runner, oracle_layer, say
from test_gpu_layer import run_and_check
from workloads import WORKLOADS, Workload, bf16_bits_to_f32

pytestmark = pytest.mark.gpu

SHAPES = [
    ("ragged-small", 2, 5, 128, 256, 333, None, 5, 5),
    ("one-token", 1, 4, 128, 128, 1, None, 2, 2),
    ("tile-edges", 1, 3, 256, 384, 128 * 3 + 1, None, 3, 3),
    ("waves-S3-W2", 3, 7, 128, 256, 500, 1.1, 3, 2),
    ("thrash-S1-W1", 2, 6, 128, 128, 200, 1.0, 1, 1),
    ("big-expert", 1, 4, 256, 512, 1500, 2.0, 4, 4),
    ("E256", 1, 256, 128, 128, 4000, 0.8, 48, 24),
    ("deep-K", 1, 9, 512, 1024, 777, 1.0, 9, 9),
]


@pytest.mark.parametrize("name,L,E,d,F,T,zipf,S,W", SHAPES)
def test_fused_small_shapes_against_oracle(name, L, E, d, F, T, zipf, S, W):
    say(f"fused layer parity: {name}")
    err = run_and_check(Workload(200 + len(name), name, L, E, d, F, T, zipf, S, W), reps=2, fused=True)
    say(f"  max rel err {err:.3e}")


def test_fused_config0():
    say("fused layer parity: config 0")
    run_and_check(WORKLOADS[0], reps=2, fused=True)


def both_paths(wl, layers):
    """y bits of the given layers from the separate-pass path and from the fused path."""
    out = []
    for fused in (False, True):
        r = make_runner(wl)
        r.ctx.set_fusion(fused)
        ins = [layer_inputs(wl, l) for l in layers]
        plans = r.plan_all([i[1] for i in ins], layers)
        dev = [r.to_device(*i) for i in ins]
        for d in dev:
            d[3].fill_(7.0)                                   # every row must be overwritten
        torch.cuda.synchronize()
        r.run(plans, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], [d[3] for d in dev])
        r.sync()
        out.append(([d[3].view(torch.uint16).cpu().numpy() for d in dev], ins, r))
    return out


@pytest.mark.parametrize("name,L,E,d,F,T,zipf,S,W", SHAPES[:1] + SHAPES[3:4] + SHAPES[5:])
def test_fused_equals_separate_passes_bit_for_bit(name, L, E, d, F, T, zipf, S, W):
    wl = Workload(300 + len(name), name, L, E, d, F, T, zipf, S, W)
    (ya, _, ra), (yb, _, rb) = both_paths(wl, list(range(L)))
    for l in range(L):
        assert np.array_equal(ya[l], yb[l]), f"{name} layer {l}"
    ra.close()
    rb.close()


def test_fused_paper_shape_streaming():
    """Switch-base-128 shape at full T: two layers streamed through the 32-slot pool (eight waves
    each), fused against separate passes bit for bit, sampled rows against the oracle."""
    wl = WORKLOADS[2].scaled(L=2)
    say(f"fused: {wl.name} L=2 streaming")
    (ya, ins, ra), (yb, _, rb) = both_paths(wl, [0, 1])
    rows = np.arange(0, wl.T, 97)
    for l in range(2):
        assert np.array_equal(ya[l], yb[l]), f"layer {l}"
        x_bits, ids, alpha = ins[l]
        y = bf16_bits_to_f32(yb[l])[rows]
        assert_close(y, oracle_layer(wl, rb, l, x_bits, ids, alpha, rows), f"layer {l}")
    ra.close()
    rb.close()
