"""Pins for the oracle's grouping of tokens by expert (counts, offsets, stable order) and for
the dispatch / combine row moves."""
import numpy as np
import pytest

import oracle
from golden_io import read_plan_trace
from workloads import WORKLOADS, gen_ids


@pytest.mark.parametrize("seed,T,E", [(0, 1, 1), (1, 17, 3), (2, 300, 8), (3, 1000, 64), (4, 777, 256)])
def test_against_numpy_library_routines(seed, T, E):
    ids = np.random.default_rng(seed).integers(0, E, T).astype(np.int32)
    counts, offsets = oracle.token_counts(ids, E)
    perm, inv = oracle.stable_order(ids, E)
    assert np.array_equal(counts, np.bincount(ids, minlength=E))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(ids, minlength=E))]))
    assert np.array_equal(perm, np.argsort(ids, kind="stable"))
    assert np.array_equal(inv[perm], np.arange(T))


def test_invariants_on_zipf_ids():
    wl = WORKLOADS[2].scaled(T=3000)
    ids = gen_ids(wl, 1)
    counts, offsets = oracle.token_counts(ids, wl.E)
    perm, inv = oracle.stable_order(ids, wl.E)
    assert counts.sum() == len(ids) and offsets[0] == 0 and offsets[-1] == len(ids)
    assert sorted(perm.tolist()) == list(range(len(ids)))
    g = ids[perm]
    assert np.all(np.diff(g) >= 0)
    same = np.diff(g) == 0
    assert np.all(np.diff(perm)[same] > 0)          # token order kept inside a group
    for e in range(wl.E):
        assert np.all(g[offsets[e]:offsets[e + 1]] == e)


def test_hand_traced_example():
    E, _, _, calls = read_plan_trace()
    for c in calls:
        counts, offsets = oracle.token_counts(c["ids"], E)
        perm, inv = oracle.stable_order(c["ids"], E)
        assert counts.tolist() == c["counts"] and offsets.tolist() == c["offsets"]
        assert perm.tolist() == c["perm"] and inv.tolist() == c["inv"]


def test_empty_and_single_group():
    counts, offsets = oracle.token_counts([], 4)
    assert counts.tolist() == [0] * 4 and offsets.tolist() == [0] * 5
    perm, inv = oracle.stable_order([], 4)
    assert perm.size == 0 and inv.size == 0
    perm, inv = oracle.stable_order([2] * 9, 4)
    assert perm.tolist() == list(range(9)) and inv.tolist() == list(range(9))


def test_bad_ids_rejected():
    with pytest.raises(ValueError):
        oracle.token_counts([0, 4], 4)
    with pytest.raises(ValueError):
        oracle.token_counts([-1], 4)


def test_dispatch_then_combine_with_unit_gates_is_identity():
    rng = np.random.default_rng(11)
    T, d, E = 123, 7, 9
    x = rng.standard_normal((T, d))
    ids = rng.integers(0, E, T)
    perm, inv = oracle.stable_order(ids, E)
    xp = oracle.dispatch(x, perm)
    assert np.array_equal(xp, x[np.argsort(ids, kind="stable")])
    assert np.array_equal(oracle.combine(xp, inv, np.ones(T)), x)
    a = rng.uniform(0.1, 1, T)
    assert np.array_equal(oracle.combine(xp, inv, a), a[:, None] * x)
