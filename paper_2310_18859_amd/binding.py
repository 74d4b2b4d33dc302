"""Thin ctypes binding: one Python method per C entry point, same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

SIDA_MAX_E = 256
POLICY_FIFO, POLICY_LRU, POLICY_BELADY = 0, 1, 2
POLICIES = {"fifo": POLICY_FIFO, "lru": POLICY_LRU, "belady": POLICY_BELADY}
EAGAIN, ECLOSED = -6, -7
DEBUG_CHECK_IDS, DEBUG_POISON_SLOTS = 1, 2
K_NAMES = ("sort", "gather", "gemm1", "gemm2", "combine", "copy")

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libsida_moe.so")


class SidaError(RuntimeError):
    def __init__(self, code: int, what: str, hip: int = 0):
        super().__init__(f"{what}: {code} ({lib().sida_strerror(code).decode()})" + (f", hipError {hip}" if hip else ""))
        self.code = code
        self.hip = hip


class SidaConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("L", "E", "d_model", "d_ff", "S", "W", "max_T")]


class SidaPlan(C.Structure):
    _fields_ = [
        ("layer", C.c_int32), ("T", C.c_int32), ("E", C.c_int32),
        ("n_active", C.c_int32), ("n_waves", C.c_int32), ("first_wave", C.c_int32),
        ("epoch", C.c_uint32), ("n_miss", C.c_int32),
        ("counts", C.c_int32 * SIDA_MAX_E), ("offsets", C.c_int32 * (SIDA_MAX_E + 1)),
        ("order", C.c_int32 * SIDA_MAX_E), ("slot", C.c_int32 * SIDA_MAX_E),
        ("wave", C.c_int32 * SIDA_MAX_E), ("hit", C.c_int32 * SIDA_MAX_E),
        ("evicted_key", C.c_int32 * SIDA_MAX_E), ("wave_dep", C.c_int32 * SIDA_MAX_E),
    ]


class SidaHashConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d_model", "C", "L", "E", "top_k", "max_seq_len")]


class WsLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in
                ("counts", "offsets", "block_hist", "perm", "inv", "x_perm", "h", "y_perm", "tiles", "sink", "gate_perm", "total")]


_LIB = None


def lib():
    """The loaded library.  Raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2310_18859_amd.build` "
                          "(or __graft_entry__.build())")
    L = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sig = {
        "sida_create": (C.c_int, [C.POINTER(SidaConfig), C.POINTER(vp)]),
        "sida_destroy": (None, [vp]),
        "sida_strerror": (C.c_char_p, [C.c_int]),
        "sida_last_hip_error": (C.c_int, [vp]),
        "sida_expert_bytes": (sz, [vp]),
        "sida_workspace_bytes": (sz, [vp, i32]),
        "sida_slot_offset": (sz, [vp, i32, i32, i32]),
        "sida_workspace_layout": (C.c_int, [vp, i32, C.POINTER(WsLayout)]),
        "sida_bind_pool": (C.c_int, [vp, vp, sz]),
        "sida_bind_host_weights": (C.c_int, [vp, C.POINTER(vp)]),
        "sida_pool_reset": (C.c_int, [vp]),
        "sida_pool_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "sida_moe_plan": (C.c_int, [vp, i32, vp, i32, C.POINTER(SidaPlan)]),
        "sida_moe_plan_lookahead": (C.c_int, [vp, i32, vp, i32, vp, C.c_int64, C.POINTER(SidaPlan)]),
        "sida_set_policy": (C.c_int, [vp, i32, i32]),
        "sida_set_fusion": (C.c_int, [vp, i32]),
        "sida_set_debug": (C.c_int, [vp, i32]),
        "sida_debug_mismatch_layer": (C.c_int, [vp]),
        "sida_set_prefetch_mode": (C.c_int, [vp, i32]),
        "sida_tile_order": (C.c_int, [i32, i32, i32, i32, vp, vp]),
        "sida_hash_param_count": (sz, [C.POINTER(SidaHashConfig)]),
        "sida_hash_workspace_bytes": (sz, [C.POINTER(SidaHashConfig), i32]),
        "sida_hash_forward": (C.c_int, [C.POINTER(SidaHashConfig), vp, vp, i32, i32, vp, vp, vp, sz, vp]),
        "sida_hash_forward_static": (C.c_int, [C.POINTER(SidaHashConfig), vp, vp, i32, i32, vp, vp, vp]),
        "sida_streams_create": (C.c_int, [i32, C.POINTER(vp), C.POINTER(vp)]),
        "sida_streams_destroy": (C.c_int, [vp, vp]),
        "sida_set_top_k": (C.c_int, [vp, i32]),
        "sida_queue_push": (C.c_int, [vp, C.c_int64, vp, i32]),
        "sida_queue_close": (C.c_int, [vp]),
        "sida_queue_size": (C.c_int, [vp]),
        "sida_queue_pop_plan": (C.c_int, [vp, i32, C.POINTER(C.c_int64), C.POINTER(i32), C.POINTER(SidaPlan)]),
        "sida_expert_prefetch": (C.c_int, [vp, C.POINTER(SidaPlan), i32, vp]),
        "sida_moe_layer_forward": (C.c_int, [vp, C.POINTER(SidaPlan), vp, vp, vp, vp, vp, sz, vp, vp]),
        "sida_run_layers": (C.c_int, [vp, i32, C.POINTER(C.POINTER(SidaPlan)), C.POINTER(vp), C.POINTER(vp),
                                      C.POINTER(vp), C.POINTER(vp), vp, sz, vp, vp]),
        "sida_dispatch": (C.c_int, [vp, vp, vp, i32, vp, sz, vp]),
        "sida_grouped_ffn": (C.c_int, [vp, C.POINTER(SidaPlan), i32, vp, sz, vp]),
        "sida_combine": (C.c_int, [vp, vp, i32, vp, vp, sz, vp]),
        "sida_profile_enable": (C.c_int, [vp, i32]),
        "sida_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _LIB = L
    return L


def _ptr(t) -> int:
    """Address of a torch tensor / numpy array / raw int (0 for None)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(s) -> int:
    if s is None:
        return 0
    if isinstance(s, int):
        return s
    return s.cuda_stream


def tile_order(m_tiles: int, m_tall: int, n_tiles_n: int, long_rows: bool = False):
    """[(token tile, weight-row tile)] in the order a grouped-GEMM launch walks its output tiles
    (long_rows: an expert's second GEMM, whose weight rows are longer than the matrix is tall)."""
    n = m_tiles * n_tiles_n
    a, b = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    rc = lib().sida_tile_order(m_tiles, m_tall, n_tiles_n, int(bool(long_rows)), a, b)
    if rc:
        raise SidaError(rc, "sida_tile_order")
    return list(zip(a[:n], b[:n]))


def hash_param_count(cfg: SidaHashConfig) -> int:
    return lib().sida_hash_param_count(C.byref(cfg))


def hash_workspace_bytes(cfg: SidaHashConfig, n_tokens: int) -> int:
    return lib().sida_hash_workspace_bytes(C.byref(cfg), n_tokens)


def hash_forward(cfg: SidaHashConfig, params, x, n_seq, seq_len, ids, alpha, workspace, stream):
    rc = lib().sida_hash_forward(C.byref(cfg), _ptr(params), _ptr(x), n_seq, seq_len, _ptr(ids), _ptr(alpha),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc:
        raise SidaError(rc, "sida_hash_forward")


def hash_forward_static(cfg: SidaHashConfig, params, x, n_seq, seq_len, ids, alpha, stream):
    rc = lib().sida_hash_forward_static(C.byref(cfg), _ptr(params), _ptr(x), n_seq, seq_len, _ptr(ids), _ptr(alpha),
                                        _stream(stream))
    if rc:
        raise SidaError(rc, "sida_hash_forward_static")


def streams_create(copy_cus: int):
    """(compute_stream, copy_stream) as raw hipStream_t values; see sida_streams_create."""
    a, b = C.c_void_p(), C.c_void_p()
    rc = lib().sida_streams_create(copy_cus, C.byref(a), C.byref(b))
    if rc:
        raise SidaError(rc, "sida_streams_create")
    return a.value, b.value


def streams_destroy(compute_stream: int, copy_stream: int):
    rc = lib().sida_streams_destroy(compute_stream, copy_stream)
    if rc:
        raise SidaError(rc, "sida_streams_destroy")


class Context:
    """Owns one sida_ctx.  Methods mirror the C entry points (without the ``sida_`` prefix)."""

    def __init__(self, L, E, d_model, d_ff, S, W, max_T):
        self.cfg = SidaConfig(L, E, d_model, d_ff, S, W, max_T)
        h = C.c_void_p()
        rc = lib().sida_create(C.byref(self.cfg), C.byref(h))
        if rc:
            raise SidaError(rc, "sida_create")
        self._h = h
        self._keep = []      # keeps bound tensors / pointer tables alive

    def close(self):
        if getattr(self, "_h", None):
            lib().sida_destroy(self._h)
            self._h = None

    __del__ = close

    def _ck(self, rc, what):
        if rc:
            raise SidaError(rc, what, lib().sida_last_hip_error(self._h) if rc == -4 else 0)

    # ---- sizes
    def expert_bytes(self) -> int:
        return lib().sida_expert_bytes(self._h)

    def slot_offset(self, which, row, col) -> int:
        return lib().sida_slot_offset(self._h, which, row, col)

    def workspace_bytes(self, T) -> int:
        return lib().sida_workspace_bytes(self._h, T)

    def workspace_layout(self, T) -> WsLayout:
        out = WsLayout()
        self._ck(lib().sida_workspace_layout(self._h, T, C.byref(out)), "sida_workspace_layout")
        return out

    # ---- binding of caller-owned memory
    def bind_pool(self, pool, nbytes=None):
        nbytes = pool.numel() * pool.element_size() if nbytes is None else nbytes
        self._ck(lib().sida_bind_pool(self._h, _ptr(pool), nbytes), "sida_bind_pool")
        self._keep.append(pool)

    def bind_host_weights(self, block_ptrs, keep=None):
        n = self.cfg.L * self.cfg.E
        if len(block_ptrs) != n:
            raise ValueError(f"need {n} block pointers")
        arr = (C.c_void_p * n)(*[int(p) for p in block_ptrs])
        self._ck(lib().sida_bind_host_weights(self._h, arr), "sida_bind_host_weights")
        self._keep.append(keep)

    def pool_reset(self):
        self._ck(lib().sida_pool_reset(self._h), "sida_pool_reset")

    def pool_state(self):
        keys = (C.c_int32 * self.cfg.S)()
        cur, nw = C.c_int32(), C.c_int32()
        self._ck(lib().sida_pool_state(self._h, keys, C.byref(cur), C.byref(nw)), "sida_pool_state")
        return list(keys), cur.value, nw.value

    # ---- the three calls
    def moe_plan(self, layer, ids_host) -> SidaPlan:
        """ids_host: contiguous int32 numpy array (or CPU tensor)."""
        plan = SidaPlan()
        T = int(ids_host.shape[0])
        self._ck(lib().sida_moe_plan(self._h, layer, _ptr(ids_host) if T else 0, T, C.byref(plan)), "sida_moe_plan")
        return plan

    def moe_plan_lookahead(self, layer, ids_host, future_keys) -> SidaPlan:
        """future_keys: contiguous int32 numpy array of keys layer*E+e in the order of their next use."""
        plan = SidaPlan()
        T, n = int(ids_host.shape[0]), int(future_keys.shape[0])
        self._ck(lib().sida_moe_plan_lookahead(self._h, layer, _ptr(ids_host) if T else 0, T,
                                               _ptr(future_keys) if n else 0, n, C.byref(plan)),
                 "sida_moe_plan_lookahead")
        return plan

    def set_prefetch_mode(self, mode):
        """mode: "auto", "copy_engine" or "kernel"."""
        m = {"auto": 0, "copy_engine": 1, "kernel": 2}.get(mode, mode)
        self._ck(lib().sida_set_prefetch_mode(self._h, m), "sida_set_prefetch_mode")

    def set_top_k(self, k: int):
        self._ck(lib().sida_set_top_k(self._h, k), "sida_set_top_k")

    def set_fusion(self, on: bool):
        self._ck(lib().sida_set_fusion(self._h, 1 if on else 0), "sida_set_fusion")

    def set_debug(self, flags: int):
        """flags: DEBUG_CHECK_IDS | DEBUG_POISON_SLOTS."""
        self._ck(lib().sida_set_debug(self._h, flags), "sida_set_debug")

    def debug_mismatch_layer(self) -> int:
        return lib().sida_debug_mismatch_layer(self._h)

    def set_policy(self, policy, lookahead_batches=0):
        self._ck(lib().sida_set_policy(self._h, POLICIES.get(policy, policy), lookahead_batches), "sida_set_policy")

    # ---- hash-table queue
    def queue_push(self, tag, ids_host):
        """ids_host: contiguous int32 numpy array [L, T]."""
        assert ids_host.ndim == 2 and ids_host.shape[0] == self.cfg.L
        T = int(ids_host.shape[1])
        self._ck(lib().sida_queue_push(self._h, tag, _ptr(ids_host) if T else 0, T), "sida_queue_push")

    def queue_close(self):
        self._ck(lib().sida_queue_close(self._h), "sida_queue_close")

    def queue_size(self) -> int:
        n = lib().sida_queue_size(self._h)
        if n < 0:
            raise SidaError(n, "sida_queue_size")
        return n

    def queue_pop_plan(self, timeout_ms=0):
        """Returns (tag, T, [SidaPlan] * L); None on timeout; raises SidaError(ECLOSED) when closed and empty."""
        plans = (SidaPlan * self.cfg.L)()
        tag, T = C.c_int64(), C.c_int32()
        rc = lib().sida_queue_pop_plan(self._h, timeout_ms, C.byref(tag), C.byref(T), plans)
        if rc == EAGAIN:
            return None
        self._ck(rc, "sida_queue_pop_plan")
        return tag.value, T.value, [plans[l] for l in range(self.cfg.L)]

    def expert_prefetch(self, plan, wave, copy_stream):
        self._ck(lib().sida_expert_prefetch(self._h, C.byref(plan), wave, _stream(copy_stream)), "sida_expert_prefetch")

    def moe_layer_forward(self, plan, x, ids, alpha, y, workspace, compute_stream, copy_stream):
        self._ck(lib().sida_moe_layer_forward(self._h, C.byref(plan), _ptr(x), _ptr(ids), _ptr(alpha), _ptr(y),
                                              _ptr(workspace), workspace.numel() * workspace.element_size(),
                                              _stream(compute_stream), _stream(copy_stream)),
                 "sida_moe_layer_forward")

    def run_layers(self, plans, xs, idss, alphas, ys, workspace, compute_stream, copy_stream):
        n = len(plans)
        pp = (C.POINTER(SidaPlan) * n)(*[C.pointer(p) for p in plans])
        mk = lambda ts: (C.c_void_p * n)(*[_ptr(t) for t in ts])
        self._ck(lib().sida_run_layers(self._h, n, pp, mk(xs), mk(idss), mk(alphas), mk(ys), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream(compute_stream), _stream(copy_stream)), "sida_run_layers")

    # ---- single stages
    def dispatch(self, x, ids, T, workspace, stream):
        self._ck(lib().sida_dispatch(self._h, _ptr(x), _ptr(ids), T, _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)), "sida_dispatch")

    def grouped_ffn(self, plan, wave, workspace, stream):
        self._ck(lib().sida_grouped_ffn(self._h, C.byref(plan), wave, _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
                 "sida_grouped_ffn")

    def combine(self, alpha, T, y, workspace, stream):
        self._ck(lib().sida_combine(self._h, _ptr(alpha), T, _ptr(y), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)), "sida_combine")

    # ---- timing
    def profile_enable(self, on: bool):
        self._ck(lib().sida_profile_enable(self._h, 1 if on else 0), "sida_profile_enable")

    def profile_read(self, reset=True):
        ms = (C.c_double * len(K_NAMES))()
        n = (C.c_int64 * len(K_NAMES))()
        self._ck(lib().sida_profile_read(self._h, ms, n, 1 if reset else 0), "sida_profile_read")
        return {k: (ms[i], n[i]) for i, k in enumerate(K_NAMES)}
