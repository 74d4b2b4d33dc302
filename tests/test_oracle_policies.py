"""Pins for the oracle's replacement policies beyond first-in-first-out and for its serving loop
(Algorithm 1 over a queue of hash tables; the footnote of Section 4.3 allows other strategies)."""
from collections import OrderedDict
from functools import lru_cache

import numpy as np
import pytest

import oracle
from golden_io import read_serve_trace

# The page-reference string most operating-systems textbooks use to compare replacement
# policies with three frames: optimal replacement takes 9 faults, least-recently-used 12,
# first-in-first-out 15.
TEXTBOOK = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]
TEXTBOOK_FAULTS = {"belady": 9, "lru": 12, "fifo": 15}


def misses(plans):
    return sum(p.hit[e] == 0 for p in plans for e in p.order)


@pytest.mark.parametrize("policy", ["fifo", "lru", "belady"])
def test_textbook_reference_string(policy):
    st = oracle.PoolState(8, 3, policy)
    plans = [st.plan_layer(0, [page], 1, TEXTBOOK[i + 1:]) for i, page in enumerate(TEXTBOOK)]
    assert misses(plans) == TEXTBOOK_FAULTS[policy]


def lru_model(E, S, calls):
    """Least-recently-used cache written the textbook way (an ordered dict, most recent last)."""
    cache, free, out = OrderedDict(), list(range(S)), []
    for layer, ids in calls:
        res = []
        for k in oracle.first_appearance(ids, E):
            key = layer * E + k
            if key in cache:
                cache.move_to_end(key)
                res.append((k, 1, -1, cache[key]))
                continue
            if free:
                s, ev = free.pop(0), -1
            else:
                ev, s = cache.popitem(last=False)
            cache[key] = s
            res.append((k, 0, ev, s))
        out.append(res)
    return out


@pytest.mark.parametrize("seed", range(40))
def test_lru_matches_an_ordered_dict_model(seed):
    rng = np.random.default_rng(300 + seed)
    E = int(rng.integers(1, 7))
    S = int(rng.integers(E, E + 5))          # a layer always fits in one wave: W = S >= E
    L = int(rng.integers(1, 4))
    calls = [(int(rng.integers(0, L)), rng.integers(0, E, int(rng.integers(0, 10))).tolist()) for _ in range(12)]
    st = oracle.PoolState(E, S, "lru")
    for (layer, ids), want in zip(calls, lru_model(E, S, calls)):
        p = st.plan_layer(layer, ids, S)
        assert [(e, p.hit[e], p.evicted_key[e], p.slot[e]) for e in p.order] == want
        assert p.n_waves == (1 if ids else 0)


def fewest_loads(E, S, calls):
    """Exhaustive search: the smallest number of loads any replacement choice can reach when every
    layer's experts must all be resident while the layer runs (one wave per layer)."""
    seq = [[layer * E + e for e in oracle.first_appearance(ids, E)] for layer, ids in calls]

    @lru_cache(maxsize=None)
    def go(c, i, resident, pinned):
        if c == len(seq):
            return 0
        if i == len(seq[c]):
            return go(c + 1, 0, resident, frozenset())
        key = seq[c][i]
        if key in resident:
            return go(c, i + 1, resident, pinned | {key})
        if len(resident) < S:
            return 1 + go(c, i + 1, resident | {key}, pinned | {key})
        return 1 + min(go(c, i + 1, (resident - {v}) | {key}, pinned | {key}) for v in resident - pinned)

    return go(0, 0, frozenset(), frozenset())


@pytest.mark.parametrize("seed", range(60))
def test_belady_reaches_the_exhaustive_optimum(seed):
    rng = np.random.default_rng(500 + seed)
    E = int(rng.integers(2, 5))
    L = int(rng.integers(1, 3))
    S = int(rng.integers(E, E + 2))          # one wave per layer
    calls = [(int(rng.integers(0, L)), rng.integers(0, E, int(rng.integers(1, 6))).tolist()) for _ in range(9)]
    keys = [[layer * E + e for e in oracle.first_appearance(ids, E)] for layer, ids in calls]
    best = fewest_loads(E, S, calls)
    got = {}
    for policy in ("fifo", "lru", "belady"):
        st = oracle.PoolState(E, S, policy)
        plans = []
        for c, (layer, ids) in enumerate(calls):
            future = [k for later in keys[c + 1:] for k in later]
            plans.append(st.plan_layer(layer, ids, S, future))
        got[policy] = misses(plans)
    assert got["belady"] == best
    assert got["fifo"] >= best and got["lru"] >= best


@pytest.mark.parametrize("policy", ["lru", "belady"])
@pytest.mark.parametrize("seed", range(25))
def test_wave_invariants_hold_for_every_policy(policy, seed):
    rng = np.random.default_rng(700 + seed)
    E = int(rng.integers(1, 20))
    S = int(rng.integers(1, 10))
    W = int(rng.integers(1, S + 1))
    st = oracle.PoolState(E, S, policy)
    calls = [(int(rng.integers(0, 3)), rng.integers(0, E, int(rng.integers(0, 40))).tolist()) for _ in range(10)]
    keys = [[layer * E + e for e in oracle.first_appearance(ids, E)] for layer, ids in calls]
    holder, g_prev, resident = {}, 0, set()
    for c, (layer, ids) in enumerate(calls):
        future = [k for later in keys[c + 1:c + 4] for k in later]
        p = st.plan_layer(layer, ids, W, future)
        assert sorted(p.order) == sorted(set(ids))
        if not ids:
            assert p.n_waves == 0 and st.g == g_prev
            continue
        assert p.first_wave == g_prev and st.g == g_prev + p.n_waves
        waves = [p.wave[e] for e in p.order]
        assert waves == sorted(waves) and set(waves) == set(range(p.first_wave, st.g))
        for w in range(p.first_wave, st.g):
            members = [e for e in p.order if p.wave[e] == w]
            slots = [p.slot[e] for e in members]
            assert 1 <= len(members) <= W and len(set(slots)) == len(slots)
            need = max([holder[p.slot[e]] for e in members if p.hit[e] == 0 and p.slot[e] in holder], default=-1)
            assert p.wave_dep[w - p.first_wave] == need
            for e in members:
                holder[p.slot[e]] = w
        for e in p.order:                              # hits are resident keys, loads evict what was there
            key = layer * E + e
            if p.hit[e] == 1:
                assert key in resident and p.evicted_key[e] == -1
            else:
                assert key not in resident
                if p.evicted_key[e] != -1:
                    resident.discard(p.evicted_key[e])
                resident.add(key)
        assert resident == {k for k in st.slot_key if k != -1}
        g_prev = st.g


def test_hand_traced_serving_loop():
    head, batches = read_serve_trace()
    E, S, W = head["E"], head["S"], head["W"]
    tables = [[c["ids"] for c in b] for b in batches]
    # the oracle exposes the loop as a whole; re-run it batch by batch to look at the state in between
    st = oracle.PoolState(E, S, head["policy"])
    for i, b in enumerate(batches):
        plans = oracle.serve_plans_step(st, tables, i, W, head["lookahead"])
        for p, c in zip(plans, b):
            got = [(e, p.slot[e], p.wave[e], p.hit[e], p.evicted_key[e]) for e in p.order]
            assert got == c["entries"]
            assert p.wave_dep == c["wave_dep"]
        assert st.slot_key == b[-1]["slot_key"] and st.g == b[-1]["g"]
    fifo = oracle.serve_plans(oracle.PoolState(E, S, "fifo"), tables, W, head["lookahead"])
    assert misses([p for b in fifo for p in b]) == head["fifo_misses"]


@pytest.mark.parametrize("seed", range(10))
def test_serving_loop_without_lookahead_is_layer_by_layer_fifo(seed):
    rng = np.random.default_rng(900 + seed)
    E, L, S, W = 6, 3, 5, 2
    tables = [[rng.integers(0, E, 7).tolist() for _ in range(L)] for _ in range(5)]
    a = oracle.serve_plans(oracle.PoolState(E, S), tables, W, 0)
    st = oracle.PoolState(E, S)
    for plans, table in zip(a, tables):
        for l, ids in enumerate(table):
            q = st.plan_layer(l, ids, W)
            p = plans[l]
            assert (p.order, p.slot, p.wave, p.hit, p.evicted_key, p.wave_dep) == (q.order, q.slot, q.wave, q.hit, q.evicted_key, q.wave_dep)


@pytest.mark.parametrize("seed", range(10))
def test_more_lookahead_never_hurts_belady_on_single_wave_layers(seed):
    rng = np.random.default_rng(1000 + seed)
    E, L, S = 5, 2, 6
    tables = [[rng.integers(0, E, 4).tolist() for _ in range(L)] for _ in range(8)]
    full = misses([p for b in oracle.serve_plans(oracle.PoolState(E, S, "belady"), tables, S, len(tables)) for p in b])
    calls = [(l, ids) for t in tables for l, ids in enumerate(t)]
    assert full == fewest_loads(E, S, calls)
    for look in (0, 1, 3):
        part = misses([p for b in oracle.serve_plans(oracle.PoolState(E, S, "belady"), tables, S, look) for p in b])
        assert part >= full
