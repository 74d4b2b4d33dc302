"""GPU parity of the whole layer path (plan -> prefetch -> sort/gather -> grouped FFN -> combine)
against the oracle, through the C ABI, at sizes the oracle finishes in seconds."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_18859_amd as sm
from gpu_util import (assert_close, bf16_tensor_to_f32, layer_inputs, make_runner, oracle_layer, say)
from workloads import WORKLOADS, Workload, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def slot_order(block, d, F):
    """An expert's host block (W_in [F, d] then W_out [d, F], row-major) in the order a pool slot
    keeps it: per matrix [R, K], stripes of 32 rows; inside a stripe the 8-element pieces are
    stored piece-major, row-minor - written here with reshapes only."""
    out = []
    for m, (R, K) in ((block[:F * d], (F, d)), (block[F * d:], (d, F))):
        pieces = m.reshape(R // 32, 32, K // 8, 8)            # [stripe, row in stripe, piece, element]
        out.append(pieces.transpose(0, 2, 1, 3).reshape(-1))  # [stripe, piece, row in stripe, element]
    return np.concatenate(out)


def run_and_check(wl, reps=1, T_of=None, check_plan=True, fused=False, prefetch=None):
    """Runs all layers `reps` times through sida_run_layers and checks every layer's y, its sort
    outputs and its plan against the oracle."""
    r = make_runner(wl)
    r.ctx.set_fusion(fused)
    if prefetch:
        r.ctx.set_prefetch_mode(prefetch)
    st = oracle.PoolState(wl.E, wl.S)
    worst = 0.0
    for rep in range(reps):
        ins = [layer_inputs(wl, l, None if T_of is None else T_of(l, rep)) for l in range(wl.L)]
        plans = r.plan_all([i[1] for i in ins])
        dev = [r.to_device(*i) for i in ins]
        r.run(plans, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], [d[3] for d in dev])
        r.sync()
        for l in range(wl.L):
            x_bits, ids, alpha = ins[l]
            op = st.plan_layer(l, ids, wl.W)
            p = plans[l]
            if check_plan:
                assert list(p.order)[:p.n_active] == op.order
                assert list(p.slot)[:wl.E] == op.slot and list(p.wave)[:wl.E] == op.wave
                assert list(p.hit)[:wl.E] == op.hit and list(p.wave_dep)[:p.n_waves] == op.wave_dep
            y = bf16_tensor_to_f32(dev[l][3])
            ref = oracle_layer(wl, r, l, x_bits, ids, alpha)
            worst = max(worst, assert_close(y, ref, f"{wl.name} rep {rep} layer {l}"))
    r.close()
    return worst


def test_config0_switch8_T256():
    say("layer parity: config 0 (E=8, d=768, F=3072, T=256, all resident)")
    err = run_and_check(WORKLOADS[0], reps=2)
    say(f"  max rel err {err:.3e}")


@pytest.mark.parametrize("name,L,E,d,F,T,zipf,S,W", [
    ("ragged-small", 2, 5, 128, 256, 333, None, 5, 5),
    ("one-token", 1, 4, 128, 128, 1, None, 2, 2),
    ("tile-edges", 1, 3, 256, 384, 128 * 3 + 1, None, 3, 3),
    ("waves-S3-W2", 3, 7, 128, 256, 500, 1.1, 3, 2),
    ("thrash-S1-W1", 2, 6, 128, 128, 200, 1.0, 1, 1),
    ("S2-W1", 2, 6, 128, 256, 257, 0.8, 2, 1),
    ("S2-W2", 2, 6, 128, 256, 257, 0.8, 2, 2),
    ("big-expert", 1, 4, 256, 512, 1500, 2.0, 4, 4),
    ("E256", 1, 256, 128, 128, 4000, 0.8, 48, 24),
])
def test_small_shapes(name, L, E, d, F, T, zipf, S, W):
    say(f"layer parity: {name}")
    wl = Workload(100 + len(name), name, L, E, d, F, T, zipf, S, W)
    err = run_and_check(wl, reps=2)
    say(f"  max rel err {err:.3e}")


@pytest.mark.parametrize("prefetch,fused", [("kernel", True), ("copy_engine", False)])
@pytest.mark.parametrize("name,E,d,F,T,zipf,S,W", [
    # the largest d_model and d_ff the library takes (K loops of 64 steps, 8 KiB rows; in copy-engine
    # mode the in-place slot re-ordering at its widest); fewer slots than experts, so slots are reloaded
    ("widest-rows", 3, 4096, 4096, 150, None, 2, 1),
    # K not a multiple of 256 (two K-steps of prefetch), N not a multiple of 256 (128-wide tiles only)
    ("odd-strides", 5, 384, 640, 300, 1.0, 5, 5),
])
def test_dimension_limits(name, E, d, F, T, zipf, S, W, prefetch, fused):
    say(f"layer parity: {name} prefetch={prefetch} fused={fused}")
    wl = Workload(120 + len(name), name, 1, E, d, F, T, zipf, S, W)
    err = run_and_check(wl, reps=2, fused=fused, prefetch=prefetch)
    say(f"  max rel err {err:.3e}")


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,E,d,F,T,zipf,rows_per_tile", [
    # most experts have at most 64 tokens, the largest several hundred: 64-row tiles, several per expert
    ("short-tiles", 40, 256, 512, 1500, 1.0, 64),
    ("short-tiles-wide", 48, 768, 3072, 1700, 1.1, 64),      # both GEMMs take 256-wide tiles
    # about 190 tokens per expert: 128-row tiles
    ("tall-tiles", 8, 256, 512, 1500, None, 128),
])
def test_both_tile_heights(name, E, d, F, T, zipf, rows_per_tile, fused):
    """The grouped GEMMs cut an expert's rows into tiles of 64 or 128 rows depending on the token
    counts of the layer; checks the descriptors the device built and the layer output for each."""
    say(f"layer parity: {name} fused={fused}")
    wl = Workload(140 + len(name), name, 1, E, d, F, T, zipf, E, E)
    r = make_runner(wl)
    r.ctx.set_fusion(fused)
    x_bits, ids, alpha = layer_inputs(wl, 0)
    x, i, a, y = r.to_device(x_bits, ids, alpha)
    plan = r.ctx.moe_plan(0, ids)
    r.ctx.moe_layer_forward(plan, x, i, a, y, r.workspace, r.compute, r.copy)
    r.sync()
    counts = np.bincount(ids, minlength=E)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    n_tiles = int(((counts + rows_per_tile - 1) // rows_per_tile).sum())
    tiles = r.region(T, "tiles", torch.int32, (n_tiles, 4)).cpu().numpy()      # slot, row0, rows, expert
    assert tiles[:, 2].max() == rows_per_tile and tiles[:, 2].min() >= 1
    covered = np.zeros(T, np.int32)
    for slot, row0, rows, e in tiles:
        assert offsets[e] <= row0 and row0 + rows <= offsets[e + 1] and (row0 - offsets[e]) % rows_per_tile == 0
        assert slot == plan.slot[e]
        covered[row0:row0 + rows] += 1
    assert np.all(covered == 1)
    ref = oracle_layer(wl, r, 0, x_bits, ids, alpha)
    err = assert_close(bf16_tensor_to_f32(y), ref, name)
    say(f"  max rel err {err:.3e}")
    r.close()


def test_varying_T_including_empty_layers():
    say("layer parity: T changes per call, some calls empty")
    wl = Workload(120, "varT", 3, 6, 128, 256, 300, 1.0, 4, 2)
    sizes = {(0, 0): 300, (1, 0): 0, (2, 0): 17, (0, 1): 1, (1, 1): 129, (2, 1): 0}
    run_and_check(wl, reps=2, T_of=lambda l, rep: sizes[(l, rep)])


def test_single_expert_is_a_dense_ffn():
    say("layer parity: E=1")
    run_and_check(Workload(130, "dense", 1, 1, 256, 512, 700, None, 1, 1))


def test_identity_experts_unit_gates_bit_exact():
    say("identity experts")
    d, T, E = 128, 999, 5
    wl = Workload(131, "identity", 1, E, d, d, T, None, E, E)
    r = make_runner(wl)
    eye = f32_to_bf16_bits(np.eye(d, dtype=np.float32)).reshape(-1)
    hw = r.host_weights.numpy()
    for e in range(E):
        hw[e, :d * d] = eye
        hw[e, d * d:] = eye
    rng = np.random.default_rng(0)
    x_bits = f32_to_bf16_bits(np.abs(rng.standard_normal((T, d))).astype(np.float32))
    ids = rng.integers(0, E, T).astype(np.int32)
    x, i, a, y = r.to_device(x_bits, ids, np.ones(T, np.float32))
    plan = r.ctx.moe_plan(0, ids)
    r.ctx.moe_layer_forward(plan, x, i, a, y, r.workspace, r.compute, r.copy)
    r.sync()
    assert np.array_equal(y.view(torch.uint16).cpu().numpy(), x_bits)
    r.close()


def test_replay_with_large_pool_hits_everything_and_repeats_y():
    say("replay: second pass all hits")
    wl = Workload(132, "replay", 3, 8, 128, 256, 400, 1.0, 24, 8)
    r = make_runner(wl)
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    outs = []
    for rep in range(2):
        plans = r.plan_all([i[1] for i in ins])
        assert all((p.n_miss == 0) == (rep == 1) for p in plans)
        dev = [r.to_device(*i) for i in ins]
        r.run(plans, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], [d[3] for d in dev])
        r.sync()
        outs.append([d[3].view(torch.uint16).cpu().numpy() for d in dev])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    r.close()


def test_explicit_prefetch_then_forward_and_order_errors():
    say("explicit prefetch / ordering errors")
    wl = Workload(133, "order", 2, 6, 128, 128, 100, None, 6, 3)
    r = make_runner(wl)
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    plans = r.plan_all([i[1] for i in ins])
    dev = [r.to_device(*i) for i in ins]
    with pytest.raises(sm.SidaError) as e:               # layer 1 before layer 0
        r.ctx.moe_layer_forward(plans[1], *dev[1], r.workspace, r.compute, r.copy)
    assert e.value.code == -3
    with pytest.raises(sm.SidaError) as e:               # wave 1 before wave 0
        r.ctx.expert_prefetch(plans[0], 1, r.copy)
    assert e.value.code == -3
    small = torch.zeros(256, dtype=torch.uint8, device=r.dev)
    with pytest.raises(sm.SidaError) as e:
        r.ctx.moe_layer_forward(plans[0], *dev[0], small, r.compute, r.copy)
    assert e.value.code == -2
    r.ctx.expert_prefetch(plans[0], 0, r.copy)           # the caller may prefetch ahead itself
    r.ctx.expert_prefetch(plans[0], 0, r.copy)           # ... twice is a no-op
    for l in range(wl.L):
        r.ctx.moe_layer_forward(plans[l], *dev[l], r.workspace, r.compute, r.copy)
    r.sync()
    for l in range(wl.L):
        ref = oracle_layer(wl, r, l, *ins[l])
        assert_close(bf16_tensor_to_f32(dev[l][3]), ref, f"layer {l}")
    with pytest.raises(sm.SidaError) as e:               # a plan is forwarded once
        r.ctx.moe_layer_forward(plans[0], *dev[0], r.workspace, r.compute, r.copy)
    assert e.value.code == -3
    r.close()


@pytest.mark.parametrize("mode", ["copy_engine", "kernel"])
def test_prefetch_by_copy_engine_and_by_kernel(mode):
    say(f"prefetch mode {mode}")
    wl = Workload(140, "prefetch-modes", 3, 9, 256, 512, 700, 1.0, 4, 2)
    r = make_runner(wl)
    r.ctx.set_prefetch_mode(mode)
    worst = 0.0
    for rep in range(2):
        ins = [layer_inputs(wl, l) for l in range(wl.L)]
        plans = r.plan_all([i[1] for i in ins])
        assert sum(p.n_miss for p in plans) > wl.S                # slots are reused within the pass
        dev = [r.to_device(*i) for i in ins]
        r.run(plans, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], [d[3] for d in dev])
        r.sync()
        for l in range(wl.L):
            x_bits, ids, alpha = ins[l]
            y = bf16_tensor_to_f32(dev[l][3])
            worst = max(worst, assert_close(y, oracle_layer(wl, r, l, x_bits, ids, alpha), f"{mode} rep {rep} layer {l}"))
    # the pool holds exactly what the plan says: every slot is its expert's host block in the
    # documented slot order (stripes of 32 rows, 16-byte pieces piece-major inside a stripe)
    keys, _, _ = r.ctx.pool_state()
    hw = r.host_weights.numpy()
    pool = r.pool.view(torch.uint16).reshape(wl.S, -1).cpu().numpy()
    for s, key in enumerate(keys):
        if key >= 0:
            assert np.array_equal(pool[s], slot_order(hw[key], wl.d_model, wl.d_ff)), f"slot {s}"
    # ... and sida_slot_offset names the same places
    rng = np.random.default_rng(3)
    s0 = next(s for s, k in enumerate(keys) if k >= 0)
    for which, (R, K) in enumerate(((wl.d_ff, wl.d_model), (wl.d_model, wl.d_ff))):
        for _ in range(50):
            row, col = int(rng.integers(R)), int(rng.integers(K))
            off = r.ctx.slot_offset(which, row, col)
            assert off % 2 == 0 and pool[s0][off // 2] == hw[keys[s0]][which * wl.d_model * wl.d_ff + row * K + col]
    assert r.ctx.slot_offset(0, wl.d_ff, 0) == 2 ** 64 - 1 and r.ctx.slot_offset(2, 0, 0) == 2 ** 64 - 1
    r.close()
    say(f"  max rel err {worst:.3e}")
