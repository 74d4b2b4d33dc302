"""GPU parity in the launch configuration bench.py's `resident` legs time: a pool of L*E slots and
waves of E experts, so that after a first pass every expert is a hit and each GEMM of a layer is ONE
launch over all activated experts (128 or 256 of them, a few hundred token tiles of both kinds -
experts with thousands of tokens beside experts with a few dozen).  Whole layers, every row,
against the oracle; the separate-pass path, the fused path and three experts per token."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, bf16_tensor_to_f32, layer_inputs, oracle_layer, say
from paper_2310_18859_amd.runner import MoERunner
from workloads import WORKLOADS, fill_host_weights, gen_gate, gen_ids, gen_x

pytestmark = pytest.mark.gpu


def resident_runner(wl):
    """As bench.py builds its resident runner."""
    r = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, wl.L * wl.E, wl.E, wl.T)
    fill_host_weights(wl, r.alloc_host_weights())
    assert r.copy_cus == 0                                 # every compute unit for the GEMMs
    return r


def run_pass(r, ins):
    plans = r.plan_all([i[1] for i in ins])
    dev = [r.to_device(*i) for i in ins]
    for d in dev:
        d[3].fill_(7.0)                                    # every row of y must be overwritten
    torch.cuda.synchronize()
    r.run(plans, [d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev], [d[3] for d in dev])
    r.sync()
    return plans, dev


def check_sort(r, wl, ids, T):
    """The sort left in the workspace by the last layer of a pass: bit-exact."""
    perm = np.argsort(ids, kind="stable").astype(np.int32)
    inv = np.empty(T, np.int32)
    inv[perm] = np.arange(T, dtype=np.int32)
    assert np.array_equal(r.region(T, "counts", torch.int32, (wl.E,)).cpu().numpy(), np.bincount(ids, minlength=wl.E))
    assert np.array_equal(r.region(T, "perm", torch.int32, (T,)).cpu().numpy(), perm)
    assert np.array_equal(r.region(T, "inv", torch.int32, (T,)).cpu().numpy(), inv)


def reaches_alternating_order(ids, E, tile_m):
    """Whether a one-launch GEMM over these tokens walks its tiles in the order that alternates blocks
    of many-token tiles with runs of few-token tiles on every XCD (csrc/tile_order.h: groups of gm
    token tiles, at least two complete rounds of 8 groups of either kind)."""
    per = [-(-int(c) // tile_m) for c in np.bincount(ids, minlength=E) if c > 0]
    m_tiles, m_tall = sum(per), sum(t for t in per if t > 1)
    gm, slack = 4, max(m_tiles // 16, m_tiles % 32)        # the group height, chosen as tile_group_height does
    for h in (8, 16):
        covered, left = (m_tall // (8 * h)) * 8 * h, m_tiles % (8 * h)
        if covered > 0 and covered * 10 >= (m_tall // 32) * 32 * 9 and left <= slack:
            gm = h
    n_many = (m_tall // gm) // 8
    return min(n_many, (m_tiles // gm) // 8 - n_many) >= 2


def check_resident(wl, whole_layers, with_top_k=False):
    say(f"resident launch shape: {wl.name} L={wl.L} E={wl.E} d={wl.d_model} F={wl.d_ff} T={wl.T}, pool of {wl.L * wl.E} slots")
    r = resident_runner(wl)
    say("  host weights ready")
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    plans, _ = run_pass(r, ins)                            # loads every activated expert
    assert all(p.n_waves == 1 for p in plans)
    # the layers that are checked row by row run the tile order with both kinds of tiles mixed
    for l in set(whole_layers[False]) | set(whole_layers[True]):
        assert reaches_alternating_order(ins[l][1], wl.E, 128), f"layer {l}"
    sample = np.arange(0, wl.T, 61)
    outs = {}
    for fused in (False, True):
        r.ctx.set_fusion(fused)
        plans, dev = run_pass(r, ins)
        assert sum(p.n_miss for p in plans) == 0 and all(p.n_waves == 1 for p in plans)
        check_sort(r, wl, ins[-1][1], wl.T)
        worst = 0.0
        for l in range(wl.L):
            x_bits, ids, alpha = ins[l]
            y = bf16_tensor_to_f32(dev[l][3])
            assert np.isfinite(y).all()
            if l in whole_layers[fused]:                   # every row of the layer
                ref = oracle_layer(wl, r, l, x_bits, ids, alpha)
                worst = max(worst, assert_close(y, ref, f"{wl.name} resident fused={fused} layer {l} (all rows)"))
            else:
                ref = oracle_layer(wl, r, l, x_bits, ids, alpha, rows=sample)
                worst = max(worst, assert_close(y[sample], ref, f"{wl.name} resident fused={fused} layer {l}"))
        outs[fused] = [d[3].view(torch.uint16).cpu().numpy() for d in dev]
        say(f"  fused={fused}: all hits, worst rel err {worst:.3e}")
    for l in range(wl.L):                                  # the two paths do the same arithmetic
        assert np.array_equal(outs[False][l], outs[True][l]), f"layer {l}: fused != separate passes"
    if with_top_k:                                         # as bench.py's top_k leg: T/3 tokens, 3 experts each
        k, hw = 3, r.host_weights.numpy()
        tok = wl.T // k
        r.ctx.set_top_k(k)
        ins_k = [(gen_x(wl, l, tok), gen_ids(wl, l, tok * k), gen_gate(wl, l, tok * k)) for l in range(wl.L)]
        for fused in (False, True):
            r.ctx.set_fusion(fused)
            run_pass(r, ins_k)                             # may activate experts the top-1 ids did not
            plans, dev = run_pass(r, ins_k)
            assert sum(p.n_miss for p in plans) == 0
            check_sort(r, wl, ins_k[-1][1], tok * k)
            l = 1 if fused else 0                          # one whole layer per mode
            x_bits, ids, alpha = ins_k[l]
            ref = oracle.moe_forward_topk(x_bits, ids.reshape(tok, k), alpha.reshape(tok, k),
                                          [hw[l * wl.E + e] for e in range(wl.E)], wl.d_model, wl.d_ff)
            err = assert_close(bf16_tensor_to_f32(dev[l][3]), ref, f"{wl.name} resident top-{k} fused={fused} layer {l}")
            say(f"  {k} experts per token, gather folded in={fused}: layer {l} all {tok} tokens, rel err {err:.3e}")
        r.ctx.set_top_k(1)
    r.close()


def test_resident_switch_base_128():
    check_resident(WORKLOADS[2], whole_layers={False: (0,), True: (3,)}, with_top_k=True)


def test_resident_switch_base_256():
    # two of the six layers: a layer's launches do not depend on how many layers share the pool
    check_resident(WORKLOADS[3].scaled(L=2), whole_layers={False: (0,), True: (1,)})


def test_resident_switch_large_128():
    check_resident(WORKLOADS[4].scaled(L=2), whole_layers={False: (1,), True: (0,)})


def test_rows_do_not_depend_on_their_neighbours():
    """A property that holds at any size and needs no oracle: a token's output row is a function of its own
    x row, expert id and gate only (Eq. 1), and the kernels sum over K in the same order wherever the
    row lands in a tile - so shuffling the tokens of a full-size layer shuffles y bit for bit.  Covers
    every row of the layers that the oracle only samples."""
    wl = WORKLOADS[2].scaled(L=2)
    say(f"token permutation at full size: {wl.name} T={wl.T}")
    r = resident_runner(wl)
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    run_pass(r, ins)                                       # loads every activated expert
    rng = np.random.default_rng(11)
    for fused in (True, False):
        r.ctx.set_fusion(fused)
        _, dev = run_pass(r, ins)
        y = [d[3].view(torch.uint16).cpu().numpy() for d in dev]
        shuffle = [rng.permutation(wl.T) for _ in range(wl.L)]
        ins_s = [(x[p], ids[p], a[p]) for (x, ids, a), p in zip(ins, shuffle)]
        _, dev_s = run_pass(r, ins_s)
        for l in range(wl.L):
            y_s = dev_s[l][3].view(torch.uint16).cpu().numpy()
            assert np.array_equal(y_s, y[l][shuffle[l]]), f"fused={fused} layer {l}"
    r.close()


def test_doubling_the_gates_doubles_y_exactly():
    """Another property without an oracle: y = bf16(alpha * bf16(sum)) (Eq. 1), so with every gate
    doubled - an exact operation in fp32 and in bf16 - every output doubles bit for bit, at full size,
    on the fused path and with the separate combine pass."""
    wl = WORKLOADS[3].scaled(L=1)
    say(f"gate scaling at full size: {wl.name} T={wl.T}")
    r = resident_runner(wl)
    ins = [layer_inputs(wl, 0)]
    run_pass(r, ins)
    for fused in (True, False):
        r.ctx.set_fusion(fused)
        _, dev = run_pass(r, ins)
        y = bf16_tensor_to_f32(dev[0][3])
        x, ids, alpha = ins[0]
        _, dev2 = run_pass(r, [(x, ids, (2.0 * alpha).astype(np.float32))])
        assert np.array_equal(bf16_tensor_to_f32(dev2[0][3]), 2.0 * y), f"fused={fused}"
    r.close()


@pytest.mark.parametrize("index,layers,mode", [(2, 6, "kernel"), (2, 6, "copy_engine"), (3, 2, "kernel"), (4, 2, "kernel")])
def test_streaming_through_a_small_pool_equals_resident_bit_for_bit(index, layers, mode):
    """A workload's streaming configuration (for the benchmark's: 32 slots, waves of 16 experts, 64-row
    tiles, every expert copied in while the previous wave computes) against the resident one (a slot
    per expert, one launch per layer, 128-row tiles): the same sums in the same K order, so every row of every
    layer must agree bit for bit - a slot read before its copy landed, or overwritten before its
    last reader finished, would show.  Both prefetch modes."""
    from gpu_util import make_runner
    wl = WORKLOADS[index] if layers == WORKLOADS[index].L else WORKLOADS[index].scaled(L=layers)
    say(f"streaming == resident at full size: {wl.name} ({layers} layers), prefetch by {mode}")
    ins = [layer_inputs(wl, l) for l in range(wl.L)]
    rs = make_runner(wl)                                   # the workload's own pool: S = 32, W = 16
    rs.ctx.set_prefetch_mode(mode)
    run_pass(rs, ins)
    plans, dev = run_pass(rs, ins)                         # steady state: every expert is a miss again
    assert sum(p.n_miss for p in plans) == sum(p.n_active for p in plans) and all(p.n_waves > 1 for p in plans)
    y_stream = [d[3].view(torch.uint16).cpu().numpy() for d in dev]
    hw = rs.host_weights
    rr = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, wl.L * wl.E, wl.E, wl.T)
    rr.host_weights = hw
    rr.ctx.bind_host_weights([hw.data_ptr() + i * rr.expert_bytes for i in range(wl.L * wl.E)], keep=hw)
    run_pass(rr, ins)
    plans, dev = run_pass(rr, ins)
    assert sum(p.n_miss for p in plans) == 0
    for l in range(wl.L):
        assert np.array_equal(dev[l][3].view(torch.uint16).cpu().numpy(), y_stream[l]), f"layer {l}"
    rs.close()
    rr.close()
