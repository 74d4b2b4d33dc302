"""Pins for the oracle's residency plan (Algorithm 1's inference-thread loop with a FIFO budget)."""
from collections import deque

import numpy as np
import pytest

import oracle
from golden_io import read_plan_trace, read_table2
from workloads import WORKLOADS, gen_ids


def entries(plan):
    return [(e, plan.slot[e], plan.wave[e], plan.hit[e], plan.evicted_key[e]) for e in plan.order]


def test_hand_traced_example():
    E, S, W, calls = read_plan_trace()
    st = oracle.PoolState(E, S)
    for c in calls:
        p = st.plan_layer(c["layer"], c["ids"], W)
        assert p.order == c["order"]
        assert entries(p) == c["entries"]
        assert p.wave_dep == c["wave_dep"]
        assert st.slot_key == c["slot_key"] and st.cursor == c["cursor"] and st.g == c["g"]


def queue_model(E, S, calls):
    """FIFO cache written the textbook way: a queue of resident keys in load order.
    Returns, per call, [(expert, hit, evicted_key, slot)] in first-appearance order."""
    q, where, free = deque(), {}, list(range(S))
    out = []
    for layer, ids in calls:
        seen, res = set(), []
        for k in ids:
            if k in seen:
                continue
            seen.add(k)
            key = layer * E + k
            if key in where:
                res.append((k, 1, -1, where[key]))
                continue
            if free:
                s, ev = free.pop(0), -1
            else:
                ev = q.popleft()
                s = where.pop(ev)
            q.append(key)
            where[key] = s
            res.append((k, 0, ev, s))
        out.append(res)
    return out


@pytest.mark.parametrize("seed", range(40))
def test_hits_misses_evictions_match_a_queue_model(seed):
    rng = np.random.default_rng(seed)
    E = int(rng.integers(1, 9))
    S = int(rng.integers(1, 7))
    W = int(rng.integers(1, S + 1))
    L = int(rng.integers(1, 4))
    calls = [(int(rng.integers(0, L)), rng.integers(0, E, int(rng.integers(0, 12))).tolist()) for _ in range(8)]
    model = queue_model(E, S, calls)
    st = oracle.PoolState(E, S)
    for (layer, ids), want in zip(calls, model):
        p = st.plan_layer(layer, ids, W)
        got = [(e, p.hit[e], p.evicted_key[e], p.slot[e]) for e in p.order]
        assert got == want


@pytest.mark.parametrize("seed", range(40))
def test_wave_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    E = int(rng.integers(1, 20))
    S = int(rng.integers(1, 10))
    W = int(rng.integers(1, S + 1))
    st = oracle.PoolState(E, S)
    g_prev = 0
    loaded, evicted = [], []
    slot_holder = {}                                   # slot -> (key, wave that computes it)
    for call in range(10):
        layer = int(rng.integers(0, 3))
        ids = rng.integers(0, E, int(rng.integers(0, 40))).tolist()
        p = st.plan_layer(layer, ids, W)
        assert sorted(p.order) == sorted(set(ids))     # every activated expert exactly once
        assert [e for e in range(E) if p.slot[e] >= 0] == sorted(set(ids))
        if not ids:
            assert p.n_waves == 0 and st.g == g_prev
            continue
        assert p.first_wave == g_prev and st.g == g_prev + p.n_waves
        waves = [p.wave[e] for e in p.order]
        assert waves == sorted(waves)                  # load order never goes back a wave
        assert set(waves) == set(range(p.first_wave, st.g))
        for w in range(p.first_wave, st.g):
            members = [e for e in p.order if p.wave[e] == w]
            slots = [p.slot[e] for e in members]
            assert 1 <= len(members) <= W and len(set(slots)) == len(slots)
            dep = p.wave_dep[w - p.first_wave]
            assert -1 <= dep < w
            # a load must wait for the last wave that computed from the slot it overwrites
            need = -1
            for e in members:
                if p.hit[e] == 0 and p.slot[e] in slot_holder:
                    need = max(need, slot_holder[p.slot[e]][1])
            assert dep == need
            for e in members:
                slot_holder[p.slot[e]] = (layer * E + e, w)
        for e in p.order:
            if p.hit[e] == 0:
                loaded.append(layer * E + e)
                if p.evicted_key[e] != -1:
                    evicted.append(p.evicted_key[e])
            else:
                assert p.evicted_key[e] == -1
        g_prev = st.g
    assert evicted == loaded[:len(evicted)]            # first in, first out
    assert len(loaded) - len(evicted) == sum(k != -1 for k in st.slot_key)


def test_large_pool_replay_is_all_hits():
    wl = WORKLOADS[1].scaled(T=2000)
    st = oracle.PoolState(wl.E, wl.L * wl.E)
    first = [st.plan_layer(l, gen_ids(wl, l), wl.L * wl.E) for l in range(wl.L)]
    again = [st.plan_layer(l, gen_ids(wl, l), wl.L * wl.E) for l in range(wl.L)]
    for a, b in zip(first, again):
        assert all(a.hit[e] == 0 and a.evicted_key[e] == -1 for e in a.order)
        assert all(b.hit[e] == 1 for e in b.order)
        assert [b.slot[e] for e in b.order] == [a.slot[e] for e in a.order]
        assert a.n_waves == 1 and b.n_waves == 1


def test_idle_experts_never_planned():
    st = oracle.PoolState(6, 4)
    p = st.plan_layer(0, [5, 5, 2], 4)
    assert p.order == [5, 2]
    for e in (0, 1, 3, 4):
        assert p.slot[e] == p.wave[e] == p.hit[e] == -1 and p.counts[e] == 0


def test_bad_id_leaves_state_untouched():
    st = oracle.PoolState(4, 2)
    st.plan_layer(0, [1, 2], 2)
    snap = (list(st.slot_key), st.cursor, list(st.last_use), st.g)
    with pytest.raises(ValueError):
        st.plan_layer(0, [0, 7], 2)
    assert snap == (st.slot_key, st.cursor, st.last_use, st.g)


def test_expert_block_size_matches_table2_slope():
    """Table 2's MoE sizes grow linearly in the number of experts; the slope is the size of one
    expert (two d_model x d_ff matrices, fp32) times the 12 MoE layers of Switch-base, in GiB."""
    t = read_table2()
    n = {"switch-base-8": 8, "switch-base-64": 64, "switch-base-128": 128, "switch-base-256": 256}
    wl = WORKLOADS[2]
    per_expert_gib = 12 * wl.expert_elems * 4 / 2 ** 30
    names = list(n)
    for a, b in zip(names, names[1:]):
        slope = (t[b][1] - t[a][1]) / (n[b] - n[a])
        assert abs(slope - per_expert_gib) / per_expert_gib < 2e-3
    assert wl.expert_bytes == 2 * 2 * 768 * 3072
