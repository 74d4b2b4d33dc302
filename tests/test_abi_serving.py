"""Host logic of the serving loop behind the C ABI (no GPU): replacement policies, planning with a
known future, and the hash-table queue between the two threads of Algorithm 1 (Section 3.1)."""
import threading
import time

import numpy as np
import pytest

import oracle
import paper_2310_18859_amd as sm
from golden_io import read_serve_trace
from test_abi_host import plans_equal
from test_oracle_policies import TEXTBOOK, TEXTBOOK_FAULTS
from workloads import WORKLOADS, gen_ids


@pytest.mark.parametrize("policy", ["fifo", "lru", "belady"])
def test_textbook_reference_string(policy):
    ctx = sm.Context(1, 8, 128, 128, 3, 1, 4)
    ctx.set_policy(policy)
    faults = 0
    for i, page in enumerate(TEXTBOOK):
        p = ctx.moe_plan_lookahead(0, np.array([page], dtype=np.int32), np.array(TEXTBOOK[i + 1:], dtype=np.int32))
        faults += p.n_miss
    assert faults == TEXTBOOK_FAULTS[policy]


@pytest.mark.parametrize("policy", ["fifo", "lru", "belady"])
@pytest.mark.parametrize("seed", range(30))
def test_planner_equals_oracle_for_every_policy(policy, seed):
    rng = np.random.default_rng(2000 + seed)
    E = int(rng.integers(1, 40))
    S = int(rng.integers(1, 24))
    W = int(rng.integers(1, S + 1))
    L = int(rng.integers(1, 5))
    ctx = sm.Context(L, E, 128, 128, S, W, 300)
    ctx.set_policy(policy)
    st = oracle.PoolState(E, S, policy)
    for call in range(14):
        layer = int(rng.integers(0, L))
        T = int(rng.integers(0, 300)) if call % 5 else 0
        ids = (rng.integers(0, E, T) if call % 2 else np.minimum(rng.zipf(1.4, T) - 1, E - 1)).astype(np.int32)
        future = rng.integers(0, L * E, int(rng.integers(0, 60))).astype(np.int32)
        plans_equal(ctx.moe_plan_lookahead(layer, ids, future), st.plan_layer(layer, ids, W, future.tolist()), E)
        keys, _, g = ctx.pool_state()
        assert keys == st.slot_key and g == st.g


def test_hand_traced_serving_loop():
    head, batches = read_serve_trace()
    E, S, W = head["E"], head["S"], head["W"]
    ctx = sm.Context(2, E, 128, 128, S, W, 8)
    ctx.set_policy(head["policy"], head["lookahead"])
    for i, b in enumerate(batches):                       # the whole stream is queued before the first pop
        T = max(len(c["ids"]) for c in b)
        assert all(len(c["ids"]) == T for c in b)
        ctx.queue_push(100 + i, np.array([c["ids"] for c in b], dtype=np.int32))
    assert ctx.queue_size() == len(batches)
    for i, b in enumerate(batches):
        tag, T, plans = ctx.queue_pop_plan(0)
        assert tag == 100 + i and T == len(b[0]["ids"])
        for p, c in zip(plans, b):
            got = [(e, p.slot[e], p.wave[e], p.hit[e], p.evicted_key[e]) for e in list(p.order)[:p.n_active]]
            assert got == c["entries"]
            assert list(p.wave_dep)[:p.n_waves] == c["wave_dep"]
        keys, _, g = ctx.pool_state()
        assert keys == b[-1]["slot_key"] and g == b[-1]["g"]
    assert ctx.queue_pop_plan(0) is None                  # empty, not closed: the thread would stay idle


@pytest.mark.parametrize("policy,look", [("fifo", 0), ("lru", 2), ("belady", 0), ("belady", 1), ("belady", 5)])
@pytest.mark.parametrize("seed", range(6))
def test_queue_plans_equal_the_oracle_serving_loop(policy, look, seed):
    rng = np.random.default_rng(3000 + seed)
    E, L, S, W, T = 12, 3, 9, 4, 20
    tables = [np.minimum(rng.zipf(1.3, (L, T)) - 1, E - 1).astype(np.int32) for _ in range(10)]
    ctx = sm.Context(L, E, 128, 128, S, W, T)
    ctx.set_policy(policy, look)
    for i, t in enumerate(tables):
        ctx.queue_push(i, t)
    want = oracle.serve_plans(oracle.PoolState(E, S, policy), [t.tolist() for t in tables], W, look)
    for i in range(len(tables)):
        tag, _, plans = ctx.queue_pop_plan(0)
        assert tag == i
        for p, q in zip(plans, want[i]):
            plans_equal(p, q, E)


def test_sentence_sized_batches_of_the_paper_shape():
    """Switch-base-128 layer shape, one short sequence per batch: hits across batches, and the
    three policies against the oracle at full E."""
    wl = WORKLOADS[2].scaled(T=128)
    rng = np.random.default_rng(7)
    perm = rng.permutation(wl.E)
    p = 1.0 / np.arange(1, wl.E + 1)
    p /= p.sum()
    tables = [perm[rng.choice(wl.E, (wl.L, wl.T), p=p)].astype(np.int32) for _ in range(6)]
    loads = {}
    for policy in ("fifo", "lru", "belady"):
        ctx = sm.Context(wl.L, wl.E, wl.d_model, wl.d_ff, 384, 64, wl.T)
        ctx.set_policy(policy, 4)
        for i, t in enumerate(tables):
            ctx.queue_push(i, t)
        want = oracle.serve_plans(oracle.PoolState(wl.E, 384, policy), [t.tolist() for t in tables], 64, 4)
        n = 0
        for i in range(len(tables)):
            _, _, plans = ctx.queue_pop_plan(0)
            for a, b in zip(plans, want[i]):
                plans_equal(a, b, wl.E)
            n += sum(a.n_miss for a in plans)
        loads[policy] = n
    active = sum(len(set(t[l].tolist())) for t in tables for l in range(wl.L))
    assert loads["belady"] <= loads["lru"] and loads["belady"] <= loads["fifo"] < active   # some hits


def test_queue_blocks_until_a_table_arrives_and_reports_close():
    ctx = sm.Context(1, 4, 128, 128, 2, 1, 4)
    t0 = time.perf_counter()
    assert ctx.queue_pop_plan(50) is None                 # nothing there: idle for the timeout
    assert time.perf_counter() - t0 >= 0.04

    def producer():                                       # the hash-building thread
        time.sleep(0.05)
        ctx.queue_push(7, np.array([[1, 1, 3]], dtype=np.int32))
        ctx.queue_close()

    th = threading.Thread(target=producer)
    th.start()
    tag, T, plans = ctx.queue_pop_plan(5000)
    th.join()
    assert (tag, T, plans[0].n_active, plans[0].n_miss) == (7, 3, 2, 2)
    with pytest.raises(sm.SidaError) as e:
        ctx.queue_pop_plan(0)
    assert e.value.code == sm.binding.ECLOSED
    with pytest.raises(sm.SidaError) as e:
        ctx.queue_push(8, np.array([[0]], dtype=np.int32))
    assert e.value.code == sm.binding.ECLOSED


def test_error_paths():
    ctx = sm.Context(2, 4, 128, 128, 3, 2, 8)
    with pytest.raises(sm.SidaError):
        ctx.set_policy(3)
    with pytest.raises(sm.SidaError):
        ctx.set_policy("lru", -1)
    with pytest.raises(sm.SidaError):                     # bad id: nothing queued
        ctx.queue_push(0, np.array([[0, 1], [4, 0]], dtype=np.int32))
    assert ctx.queue_size() == 0
    with pytest.raises(sm.SidaError):                     # bad future key: state untouched
        ctx.moe_plan_lookahead(0, np.array([1], dtype=np.int32), np.array([8], dtype=np.int32))
    assert ctx.pool_state()[0] == [-1, -1, -1]
    ctx.moe_plan(0, np.array([1], dtype=np.int32))
    with pytest.raises(sm.SidaError) as e:                # policy changes only on an empty pool
        ctx.set_policy("lru")
    assert e.value.code == -3
    ctx.pool_reset()
    ctx.set_policy("lru")
    for i in range(256):
        ctx.queue_push(i, np.zeros((2, 1), dtype=np.int32))
    with pytest.raises(sm.SidaError) as e:
        ctx.queue_push(256, np.zeros((2, 1), dtype=np.int32))
    assert e.value.code == -2
