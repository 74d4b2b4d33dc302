"""CPU-side tests of the C-ABI library: it loads, exports what the header declares, rejects bad
arguments, and its host planner agrees bit for bit with the oracle's Algorithm-1 simulation."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2310_18859_amd as sm
from golden_io import read_plan_trace
from workloads import WORKLOADS, gen_ids

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sida_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sida_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 18 and "sida_moe_plan" in names and "sida_moe_layer_forward" in names
    lib = ctypes.CDLL(sm.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_plan_struct_matches_header_size():
    # 8 scalars + 7 arrays of 256 + one of 257 int32
    assert ctypes.sizeof(sm.SidaPlan) == 4 * (8 + 7 * 256 + 257)


def plans_equal(p, q, E):
    assert (p.layer, p.T, p.E, p.n_active, p.n_waves, p.first_wave) == (q.layer, q.T, q.E, q.n_active, q.n_waves, q.first_wave)
    assert list(p.counts)[:E] == q.counts.tolist()
    assert list(p.offsets)[:E + 1] == q.offsets.tolist()
    assert list(p.order)[:p.n_active] == q.order
    for name in ("slot", "wave", "hit", "evicted_key"):
        assert list(getattr(p, name))[:E] == getattr(q, name), name
    assert list(p.wave_dep)[:p.n_waves] == q.wave_dep
    assert p.n_miss == sum(1 for e in q.order if q.hit[e] == 0)


def test_hand_traced_example():
    E, S, W, calls = read_plan_trace()
    ctx = sm.Context(2, E, 128, 128, S, W, 64)
    for c in calls:
        p = ctx.moe_plan(c["layer"], np.array(c["ids"], dtype=np.int32))
        got = [(e, p.slot[e], p.wave[e], p.hit[e], p.evicted_key[e]) for e in list(p.order)[:p.n_active]]
        assert got == c["entries"]
        assert list(p.wave_dep)[:p.n_waves] == c["wave_dep"]
        keys, cur, g = ctx.pool_state()
        assert keys == c["slot_key"] and cur == c["cursor"] and g == c["g"]


@pytest.mark.parametrize("seed", range(60))
def test_planner_equals_oracle_on_random_streams(seed):
    rng = np.random.default_rng(seed)
    E = int(rng.integers(1, 40))
    S = int(rng.integers(1, 24))
    W = int(rng.integers(1, S + 1))
    L = int(rng.integers(1, 5))
    ctx = sm.Context(L, E, 128, 128, S, W, 400)
    st = oracle.PoolState(E, S)
    for call in range(12):
        layer = int(rng.integers(0, L))
        T = int(rng.integers(0, 400)) if call % 5 else 0
        skew = rng.integers(0, 3)
        ids = rng.integers(0, E, T) if skew == 0 else np.minimum(rng.zipf(1.5, T) - 1, E - 1) if skew == 1 \
            else np.full(T, rng.integers(0, E))
        ids = ids.astype(np.int32)
        plans_equal(ctx.moe_plan(layer, ids), st.plan_layer(layer, ids, W), E)
        keys, cur, g = ctx.pool_state()
        assert keys == st.slot_key and cur == st.cursor and g == st.g


@pytest.mark.parametrize("wi", [1, 2, 3, 4])
def test_planner_equals_oracle_on_paper_shaped_workloads(wi):
    wl = WORKLOADS[wi]
    ctx = sm.Context(wl.L, wl.E, wl.d_model, wl.d_ff, wl.S, wl.W, wl.T)
    st = oracle.PoolState(wl.E, wl.S)
    for rep in range(2):
        for l in range(wl.L):
            ids = gen_ids(wl, l)
            plans_equal(ctx.moe_plan(l, ids), st.plan_layer(l, ids, wl.W), wl.E)
    assert ctx.pool_state() == (st.slot_key, st.cursor, st.g)


def test_pool_reset_and_stale_plans():
    ctx = sm.Context(1, 4, 128, 128, 2, 2, 16)
    p = ctx.moe_plan(0, np.array([1, 2], dtype=np.int32))
    ctx.pool_reset()
    assert ctx.pool_state() == ([-1, -1], 0, 0)
    with pytest.raises(sm.SidaError) as e:
        ctx.expert_prefetch(p, 0, None)          # plan from before the reset
    assert e.value.code == -3


def test_error_paths_leave_state_untouched():
    with pytest.raises(sm.SidaError):
        sm.Context(1, 257, 128, 128, 2, 2, 16)    # E too large
    with pytest.raises(sm.SidaError):
        sm.Context(1, 4, 100, 128, 2, 2, 16)      # d_model not a multiple of 128
    with pytest.raises(sm.SidaError):
        sm.Context(1, 4, 128, 128, 2, 3, 16)      # W > S
    ctx = sm.Context(2, 4, 128, 128, 2, 2, 16)
    ctx.moe_plan(0, np.array([1, 2], dtype=np.int32))
    before = ctx.pool_state()
    for bad in ([0, 4], [-1], [0] * 17):
        with pytest.raises(sm.SidaError) as e:
            ctx.moe_plan(0, np.array(bad, dtype=np.int32))
        assert e.value.code == -1
    with pytest.raises(sm.SidaError):
        ctx.moe_plan(2, np.array([0], dtype=np.int32))       # layer out of range
    assert ctx.pool_state() == before
    assert ctx.workspace_bytes(17) == 0 and ctx.workspace_bytes(16) > 0
    p = ctx.moe_plan(1, np.array([3], dtype=np.int32))
    with pytest.raises(sm.SidaError) as e:                    # pool and host weights not bound
        ctx.expert_prefetch(p, 0, None)
    assert e.value.code == -3
    with pytest.raises(sm.SidaError) as e:
        ctx.expert_prefetch(p, 5, None)
    assert e.value.code == -1


def test_workspace_layout_is_aligned_and_ordered():
    ctx = sm.Context(1, 64, 768, 3072, 8, 8, 5000)
    lay = ctx.workspace_layout(4999)
    offs = [lay.counts, lay.offsets, lay.block_hist, lay.perm, lay.inv, lay.x_perm, lay.h, lay.y_perm, lay.tiles, lay.sink, lay.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lay.h - lay.x_perm >= 4999 * 768 * 2 and lay.y_perm - lay.h >= 4999 * 3072 * 2
    assert lay.total == ctx.workspace_bytes(4999)
    assert ctx.expert_bytes() == 4 * 768 * 3072


def test_prefetch_mode_arguments():
    ctx = sm.Context(1, 4, 128, 128, 2, 1, 8)
    ctx.set_prefetch_mode("auto")
    ctx.set_prefetch_mode("copy_engine")
    with pytest.raises(sm.SidaError) as e:                # no pinned blocks bound: the kernel cannot read them
        ctx.set_prefetch_mode("kernel")
    assert e.value.code == -3
    with pytest.raises(sm.SidaError):
        ctx.set_prefetch_mode(3)


def test_tile_order_visits_every_tile_once():
    """The walk order of a grouped-GEMM launch (the same function the kernels use) is a bijection for
    every mix of many-token and few-token tiles, including the launches whose XCDs alternate the two."""
    rng = np.random.default_rng(5)
    shapes = [(m, mt, n) for m in (0, 1, 3, 4, 31, 32, 33, 63, 64, 65, 100, 128, 130, 204, 256, 257, 330, 384, 512)
              for mt in sorted({0, 2 if m >= 2 else 0, m // 3, m // 2, m - m % 4, m}) if mt <= m
              for n in (1, 3, 4, 6, 12, 16, 24)]
    shapes += [(int(rng.integers(1, 700)), 0, int(rng.choice([3, 6, 12, 16, 32]))) for _ in range(40)]
    for m, mt, n in shapes:
        if mt == 0 and rng.random() < 0.5 and m > 8:
            mt = int(rng.integers(0, m + 1))
        for long_rows in (False, True):
            order = sm.tile_order(m, mt, n, long_rows)
            assert len(order) == m * n
            assert sorted(order) == [(a, b) for a in range(m) for b in range(n)], (m, mt, n, long_rows)
    # cases where the mixing is active: at least two rounds (64 token tiles) of either kind
    mixed = sm.tile_order(204, 100, 12)
    plain = [(t // 12, t % 12) for t in range(204 * 12)]
    assert mixed != plain and sorted(mixed) == plain
    # many-token experts alone (8 experts x 16 token tiles): groups of 16 token tiles, so the 64 tiles an
    # XCD works on at a time share one expert's 16 token tiles and 4 weight-row tiles
    tall = sm.tile_order(128, 128, 12)
    for xcd in range(8):
        first = tall[xcd::8][:64]
        assert {a // 16 for a, _ in first} == {xcd} and len({b for _, b in first}) == 4
    # an expert's second GEMM with two rounds of either kind of tile in groups of 8 (the Switch-large
    # shape): an XCD starts with one many-token expert's 8 token tiles against all weight-row tiles
    second = sm.tile_order(328, 234, 4, True)
    assert second != sm.tile_order(328, 234, 4, False) and sorted(second) == [(t // 4, t % 4) for t in range(328 * 4)]
    assert sorted(second[0::8][:32]) == [(a, b) for a in range(8) for b in range(4)]
    assert sm.tile_order(204, 100, 6, True) == sm.tile_order(204, 100, 6, False)     # one round only: groups of 4
    with pytest.raises(sm.SidaError):
        sm.tile_order(4, 5, 3)


def test_hash_function_sizes():
    cfg = sm.SidaHashConfig(768, 128, 6, 128, 3, 512)
    C, d, L, E = 128, 768, 6, 128
    assert sm.hash_param_count(cfg) == C * d + C + 2 * (8 * C * C + 8 * C) + L * E * C + L * E
    assert sm.hash_param_count(cfg) == sum(int(np.prod(s)) for _, s in __import__("oracle.hash_fn").hash_fn.param_shapes(d, C, L, E))
    assert sm.hash_workspace_bytes(cfg, 100) >= 4 * 8 * C * 100
    assert sm.hash_param_count(sm.SidaHashConfig(768, 100, 6, 128, 3, 512)) == 0
