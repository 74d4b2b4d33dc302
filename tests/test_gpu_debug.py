"""The debug switches of the boundary: the check that a layer ran with the ids it was planned with,
and the NaN poisoning of slots before they are reloaded (the slot-reuse race between the copy and
the compute stream would then show up as NaN in y)."""
import numpy as np
import pytest
import torch

import paper_2310_18859_amd as sm
from gpu_util import assert_close, bf16_tensor_to_f32, layer_inputs, make_runner, oracle_layer, say
from paper_2310_18859_amd.binding import DEBUG_CHECK_IDS, DEBUG_POISON_SLOTS
from workloads import Workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,L,E,d,F,T,zipf,S,W", [
    ("thrash-S1-W1", 2, 6, 128, 128, 200, 1.0, 1, 1),
    ("S2-W1", 2, 6, 128, 256, 257, 0.8, 2, 1),
    ("waves-S3-W2", 3, 7, 128, 256, 500, 1.1, 3, 2),
    ("S8-W4", 3, 20, 256, 512, 3000, 1.0, 8, 4),
])
@pytest.mark.parametrize("mode", ["kernel", "copy_engine"])
def test_poisoned_slots_never_reach_the_output(name, L, E, d, F, T, zipf, S, W, mode):
    """Every slot is filled with NaNs before each reload; with a correct wave / event order no
    grouped FFN reads a slot before its copies finished, so y stays finite and right."""
    say(f"poison {name} {mode}")
    wl = Workload(700 + len(name), name, L, E, d, F, T, zipf, S, W)
    r = make_runner(wl)
    r.ctx.set_prefetch_mode(mode)
    r.ctx.set_debug(DEBUG_POISON_SLOTS | DEBUG_CHECK_IDS)
    for rep in range(3):
        ins = [layer_inputs(wl, l) for l in range(wl.L)]
        plans = r.plan_all([i[1] for i in ins])
        dev = [r.to_device(*i) for i in ins]
        r.run(plans, [d_[0] for d_ in dev], [d_[1] for d_ in dev], [d_[2] for d_ in dev], [d_[3] for d_ in dev])
        r.sync()
        for l in range(wl.L):
            x_bits, ids, alpha = ins[l]
            y = bf16_tensor_to_f32(dev[l][3])
            assert np.isfinite(y).all(), f"rep {rep} layer {l}: poison reached y"
            assert_close(y, oracle_layer(wl, r, l, x_bits, ids, alpha), f"{name} rep {rep} layer {l}")
    assert r.ctx.debug_mismatch_layer() == -1
    r.close()


def test_poison_fills_the_slot_when_nothing_overwrites_it():
    """The poison kernel itself: a wave whose host blocks are all-zero experts would leave zeros; run
    the prefetch with poisoning and look at a slot's bytes BEFORE the copy of the next wave lands is
    not observable from outside - so check the pattern through the one place that keeps it: a slot
    of a pool with more slots than the plan uses stays untouched, a used one holds its expert."""
    wl = Workload(720, "poison-pool", 1, 4, 128, 128, 64, None, 6, 6)
    r = make_runner(wl)
    r.pool.fill_(0x11)
    torch.cuda.synchronize()
    r.ctx.set_debug(DEBUG_POISON_SLOTS)
    x_bits, ids, alpha = layer_inputs(wl, 0)
    plan = r.ctx.moe_plan(0, ids)
    xd, idd, ad, yd = r.to_device(x_bits, ids, alpha)
    r.ctx.moe_layer_forward(plan, xd, idd, ad, yd, r.workspace, r.compute, r.copy)
    r.sync()
    pool = r.pool.reshape(wl.S, -1).cpu().numpy()
    used = {plan.slot[e] for e in range(wl.E) if plan.slot[e] >= 0}
    for s in range(wl.S):
        if s in used:
            assert not (pool[s] == 0x11).all()
        else:
            assert (pool[s] == 0x11).all()                   # neither poisoned nor copied
    assert np.isfinite(bf16_tensor_to_f32(yd)).all()
    r.close()


def test_ids_that_differ_from_the_plan_are_caught():
    wl = Workload(730, "id-check", 2, 9, 128, 256, 300, 1.0, 9, 9)
    r = make_runner(wl)
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    plans = r.plan_all([i[1] for i in ins])
    dev = [r.to_device(*i) for i in ins]
    other = ins[1][1].copy()
    other[:7] = (other[:7] + 1) % wl.E                        # valid ids, but not the planned ones
    bad = torch.from_numpy(other).to(r.dev)

    def run(ids1):
        r.run(plans, [d_[0] for d_ in dev], [dev[0][1], ids1], [d_[2] for d_ in dev], [d_[3] for d_ in dev])
        r.sync()

    # without the switch the mismatch goes unnoticed (status 0): that is the documented contract
    run(bad)
    assert r.ctx.debug_mismatch_layer() == -1
    r.ctx.pool_reset()
    r.ctx.set_debug(DEBUG_CHECK_IDS)
    plans = r.plan_all([i[1] for i in ins])
    run(dev[1][1])                                            # the right ids: nothing latched
    assert r.ctx.debug_mismatch_layer() == -1
    plans = r.plan_all([i[1] for i in ins])
    run(bad)                                                  # enqueued fine; the check runs on the stream
    assert r.ctx.debug_mismatch_layer() == 1
    plans = r.plan_all([i[1] for i in ins])
    with pytest.raises(sm.SidaError) as e:                    # ... and every later call refuses
        run(dev[1][1])
    assert e.value.code == -3
    r.ctx.pool_reset()                                        # clears the latch
    assert r.ctx.debug_mismatch_layer() == -1
    plans = r.plan_all([i[1] for i in ins])
    run(dev[1][1])
    for l in range(wl.L):
        x_bits, ids, alpha = ins[l]
        assert_close(bf16_tensor_to_f32(dev[l][3]), oracle_layer(wl, r, l, x_bits, ids, alpha), f"layer {l}")
    with pytest.raises(sm.SidaError):
        r.ctx.set_debug(8)
    r.close()
