"""CPU oracle for the SiDA-MoE layer hot path.  TEST INFRASTRUCTURE ONLY.

May be imported by tests/, by ``__graft_entry__.smoke()`` and by ``bench.py``'s cpu_baseline leg;
the product package never imports it and it never imports the product package.

Floating point: see ``sida_oracle.c`` (Eq. 1 of Section 2.1 with top-1 selection, expert id and
scaling factor looked up per token as in Section 3.1).  Integer parts, all plain Python loops:

* ``token_counts`` / ``stable_order``: the grouping of tokens by expert that any "invoke only the
  experts that have tokens" implementation (Section 2.3) needs.  The paper prescribes no order,
  so the only order that is unique is used: by expert id, ties by token index.
* ``PoolState.plan_layer``: the inference thread's residency step of Algorithm 1 ("for each
  MoE layer and each token: check the expert; if it is not on the GPU, move it there") under a
  GPU memory budget of S equal-sized expert slots with first-in-first-out replacement
  (Section 3.1 and Section 4.3).  Where the paper is silent the readings are: experts are
  loaded in order of first appearance in the token stream; a hit does not renew an expert's
  age; the budget is global over layers (key = layer*E + e); when more experts are needed by
  one layer than fit, the layer is cut into waves of at most W experts, and a slot may only be
  overwritten after the wave that last computed from it has finished (``wave_dep``).
* Replacement policies other than first-in-first-out (the footnote of Section 4.3 allows them):
  ``"lru"`` overwrites the expert that was loaded or hit longest ago, ``"belady"`` the expert
  whose next use lies farthest ahead in the known future - the rest of the current layer, then
  ``future_keys``, which the hash-table queue of Section 3.1 makes available (ties: the oldest
  load).  Both use empty slots first and never take a slot of the wave being assembled.
* ``serve_plans``: the inference thread's loop over a queue of hash tables (Algorithm 1,
  Section 3.1): batches are planned in arrival order, layer by layer, each layer seeing the
  later layers of its batch and the queued batches behind it as its future.

Pins: tests/test_oracle_forward.py, tests/test_oracle_sort.py, tests/test_oracle_plan.py,
tests/test_oracle_policies.py.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libsida_oracle.so")
        if not os.path.exists(path):
            from . import build as _b
            _b.build()
        lib = ctypes.CDLL(path)
        lib.sida_oracle_moe_forward.restype = ctypes.c_int
        lib.sida_oracle_moe_forward.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.sida_oracle_moe_forward_topk.restype = ctypes.c_int
        lib.sida_oracle_moe_forward_topk.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.sida_oracle_threads.restype = ctypes.c_int
        _LIB = lib
    return _LIB


def threads() -> int:
    """Number of host threads the C forward uses."""
    return int(_lib().sida_oracle_threads())


# --------------------------------------------------------------------------- layer output
def moe_forward(x_bf16, ids, alpha, blocks, d_model: int, d_ff: int) -> np.ndarray:
    """y[t] = alpha[t] * W_out[k] relu(W_in[k] x[t]),  k = ids[t]   (Eq. 1, top-1).

    x_bf16: uint16 [T, d] bf16 bit patterns.  ids: int32 [T].  alpha: float32 [T].
    blocks: sequence of E uint16 arrays of 2*d*F bf16 values, W_in [F,d] then W_out [d,F].
    Returns float32 [T, d]."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    alpha = np.ascontiguousarray(alpha, dtype=np.float32)
    T = ids.shape[0]
    assert x.shape == (T, d_model) and alpha.shape == (T,)
    keep = [np.ascontiguousarray(b, dtype=np.uint16).reshape(-1) for b in blocks]
    for b in keep:
        assert b.size == 2 * d_model * d_ff
    E = len(keep)
    ptrs = (ctypes.c_void_p * max(E, 1))(*[b.ctypes.data for b in keep])
    y = np.empty((T, d_model), dtype=np.float32)
    rc = _lib().sida_oracle_moe_forward(x.ctypes.data, ids.ctypes.data, alpha.ctypes.data,
                                        ctypes.cast(ptrs, ctypes.c_void_p), E, T, d_model, d_ff,
                                        y.ctypes.data)
    if rc != 0:
        raise ValueError("expert id out of range")
    return y


def moe_forward_topk(x_bf16, ids, alpha, blocks, d_model: int, d_ff: int) -> np.ndarray:
    """y[t] = sum_j alpha[t,j] * W_out[e] relu(W_in[e] x[t]),  e = ids[t,j]   (Eq. 1, |I| = k).

    ids: int32 [T,k].  alpha: float32 [T,k].  Otherwise as moe_forward.  Returns float32 [T, d]."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    alpha = np.ascontiguousarray(alpha, dtype=np.float32)
    assert ids.ndim == 2 and alpha.shape == ids.shape
    T, k = ids.shape
    assert x.shape == (T, d_model)
    keep = [np.ascontiguousarray(b, dtype=np.uint16).reshape(-1) for b in blocks]
    for b in keep:
        assert b.size == 2 * d_model * d_ff
    E = len(keep)
    ptrs = (ctypes.c_void_p * max(E, 1))(*[b.ctypes.data for b in keep])
    y = np.empty((T, d_model), dtype=np.float32)
    rc = _lib().sida_oracle_moe_forward_topk(x.ctypes.data, ids.ctypes.data, alpha.ctypes.data,
                                             ctypes.cast(ptrs, ctypes.c_void_p), E, T, k, d_model, d_ff,
                                             y.ctypes.data)
    if rc != 0:
        raise ValueError("expert id out of range")
    return y


# --------------------------------------------------------------------------- grouping by expert
def token_counts(ids, E: int):
    """counts[e] = number of tokens with id e; offsets = exclusive prefix sum, offsets[E] = T."""
    counts = [0] * E
    for k in ids:
        k = int(k)
        if not 0 <= k < E:
            raise ValueError("expert id out of range")
        counts[k] += 1
    offsets = [0] * (E + 1)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    return np.array(counts, dtype=np.int32), np.array(offsets, dtype=np.int32)


def stable_order(ids, E: int):
    """perm[offsets[e] + j] = the j-th smallest token index t with ids[t] == e;  inv[perm[r]] = r."""
    _, offsets = token_counts(ids, E)
    T = len(ids)
    perm = [0] * T
    inv = [0] * T
    r = 0
    for e in range(E):
        assert r == offsets[e]
        for t in range(T):
            if int(ids[t]) == e:
                perm[r] = t
                inv[t] = r
                r += 1
    return np.array(perm, dtype=np.int32), np.array(inv, dtype=np.int32)


def dispatch(x, perm):
    """x_perm[r] = x[perm[r]] (rows moved, bits untouched)."""
    x = np.asarray(x)
    out = np.empty_like(x)
    for r in range(len(perm)):
        out[r] = x[int(perm[r])]
    return out


def combine(y_perm, inv, alpha):
    """y[t] = alpha[t] * y_perm[inv[t]] in fp64 (the alpha factor of Eq. 1, back in token order)."""
    y_perm = np.asarray(y_perm, dtype=np.float64)
    out = np.empty_like(y_perm)
    for t in range(len(inv)):
        out[t] = float(alpha[t]) * y_perm[int(inv[t])]
    return out


# --------------------------------------------------------------------------- residency plan
class LayerPlan:
    """Result of planning one layer.  Arrays indexed by expert id hold -1 for idle experts."""

    def __init__(self, layer, T, E):
        self.layer, self.T, self.E = layer, T, E
        self.counts = None
        self.offsets = None
        self.order = []                 # activated experts, first-appearance order
        self.slot = [-1] * E
        self.wave = [-1] * E            # global wave index
        self.hit = [-1] * E             # 1 hit, 0 miss
        self.evicted_key = [-1] * E     # key overwritten by this expert's load, -1 if none
        self.first_wave = -1
        self.n_waves = 0
        self.wave_dep = []              # per local wave: global wave whose compute must end first, or -1

    @property
    def n_active(self):
        return len(self.order)


NEVER = 1 << 60     # "not used again" as a next-use distance


def first_appearance(ids, E: int):
    """Experts of a layer in the order Algorithm 1 meets them when it walks the tokens."""
    seen, order = [False] * E, []
    for k in ids:
        k = int(k)
        if not 0 <= k < E:
            raise ValueError("expert id out of range")
        if not seen[k]:
            seen[k] = True
            order.append(k)
    return order


class PoolState:
    """S equal-sized expert slots, shared by all layers.  policy: "fifo" (the paper's), "lru", "belady"."""

    def __init__(self, E: int, S: int, policy: str = "fifo"):
        if S < 1 or E < 1:
            raise ValueError("need S >= 1 and E >= 1")
        if policy not in ("fifo", "lru", "belady"):
            raise ValueError("unknown policy")
        self.E, self.S, self.policy = E, S, policy
        self.slot_key = [-1] * S        # layer*E + e held by each slot
        self.cursor = 0                 # fifo: next slot to overwrite == the oldest load
        self.last_use = [-1] * S        # global wave that last computed from the slot
        self.g = 0                      # next global wave index
        self.clock = 0                  # counts loads and hits
        self.loaded_at = [-1] * S       # clock value of the load that filled the slot
        self.touched_at = [-1] * S      # clock value of the slot's last load or hit

    def _victim(self, in_wave, next_use):
        """Slot to overwrite, or -1 when every slot belongs to the wave being assembled."""
        free = [s for s in range(self.S) if s not in in_wave]
        if not free:
            return -1
        for s in free:
            if self.slot_key[s] == -1:
                return s
        if self.policy == "lru":
            return min(free, key=lambda s: self.touched_at[s])
        best = free[0]
        for s in free[1:]:
            a, b = next_use(self.slot_key[s]), next_use(self.slot_key[best])
            if a > b or (a == b and self.loaded_at[s] < self.loaded_at[best]):
                best = s
        return best

    def plan_layer(self, layer: int, ids, W: int, future_keys=()) -> LayerPlan:
        E, S = self.E, self.S
        if not 1 <= W <= S:
            raise ValueError("need 1 <= W <= S")
        T = len(ids)
        plan = LayerPlan(layer, T, E)
        plan.counts, plan.offsets = token_counts(ids, E)      # raises on a bad id before any change

        # Algorithm 1: walk the tokens in order and check each token's expert.
        plan.order = first_appearance(ids, E)
        if not plan.order:
            return plan

        # next use of a resident key, seen from expert number i of this layer: the experts still
        # to come in this layer are the nearest uses, then the caller's future in its order
        place = {layer * E + e: j for j, e in enumerate(plan.order)}
        later = {}
        for j, k in enumerate(future_keys):
            later.setdefault(int(k), j)

        plan.first_wave = self.g
        deps = {self.g: -1}
        n = 0
        in_wave = set()                 # slots the current wave computes from

        def new_wave():
            nonlocal n, in_wave
            self.g += 1
            deps[self.g] = -1
            n, in_wave = 0, set()

        for i, e in enumerate(plan.order):
            key = layer * E + e

            def next_use(k):
                if place.get(k, -1) > i:
                    return place[k] - i
                return len(plan.order) + later[k] if k in later else NEVER

            s = self.slot_key.index(key) if key in self.slot_key else -1
            if s != -1:                                        # on the GPU already
                if n == W:
                    new_wave()
                plan.hit[e] = 1
            else:                                              # not on the GPU: load it
                if self.policy == "fifo":
                    if n == W or self.cursor in in_wave:
                        new_wave()
                    s = self.cursor
                    self.cursor = (self.cursor + 1) % S
                else:
                    if n == W:
                        new_wave()
                    s = self._victim(in_wave, next_use)
                    if s == -1:
                        new_wave()
                        s = self._victim(in_wave, next_use)
                plan.evicted_key[e] = self.slot_key[s]
                self.slot_key[s] = key
                self.loaded_at[s] = self.clock
                deps[self.g] = max(deps[self.g], self.last_use[s])
                plan.hit[e] = 0
            self.touched_at[s] = self.clock
            self.clock += 1
            plan.slot[e] = s
            plan.wave[e] = self.g
            in_wave.add(s)
            n += 1
            self.last_use[s] = self.g
        self.g += 1                                            # the next layer starts a new wave
        plan.n_waves = self.g - plan.first_wave
        plan.wave_dep = [deps[plan.first_wave + w] for w in range(plan.n_waves)]
        return plan


def serve_plans_step(pool: PoolState, batches, i: int, W: int, lookahead: int):
    """Plans batch i of the stream: what the inference thread does after popping hash table i
    while the `lookahead` batches behind it (fewer at the end of the stream) wait in the queue."""
    E = pool.E
    table = batches[i]
    visible = batches[i + 1:i + 1 + lookahead]
    plans = []
    for l, ids in enumerate(table):
        future = []
        for l2 in range(l + 1, len(table)):
            future += [l2 * E + e for e in first_appearance(table[l2], E)]
        for other in visible:
            for l2, ids2 in enumerate(other):
                future += [l2 * E + e for e in first_appearance(ids2, E)]
        plans.append(pool.plan_layer(l, ids, W, future))
    return plans


def serve_plans(pool: PoolState, batches, W: int, lookahead: int):
    """Plans a stream of batches the way the inference thread consumes the hash-table queue.

    batches: list of hash tables, each a list of L id arrays (one per MoE layer), in arrival order.
    Returns one list of LayerPlan per batch."""
    return [serve_plans_step(pool, batches, i, W, lookahead) for i in range(len(batches))]
