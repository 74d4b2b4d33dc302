"""Device-memory and stream plumbing around the binding: allocates the caller-owned buffers the
C ABI expects (slot pool, workspace, pinned host weights, per-layer tensors) with PyTorch and
drives plan -> prefetch -> forward.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from .binding import Context, streams_create, streams_destroy


class MoERunner:
    def __init__(self, L, E, d_model, d_ff, S, W, max_T, device="cuda:0", copy_cus=None):
        """copy_cus: compute units set aside for the copy stream (sida_streams_create).  None: 16 when
        experts have to stream through the pool (S < L*E), else 0 (plain streams, every compute unit
        for the GEMMs)."""
        if not torch.cuda.is_available():
            raise RuntimeError("MoERunner needs a GPU: the HIP path has no CPU fallback")
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.L, self.E, self.d, self.F, self.S, self.W, self.max_T = L, E, d_model, d_ff, S, W, max_T
        self.ctx = Context(L, E, d_model, d_ff, S, W, max_T)
        self.expert_bytes = self.ctx.expert_bytes()
        self.expert_elems = self.expert_bytes // 2
        self.pool = torch.zeros(S * self.expert_bytes, dtype=torch.uint8, device=self.dev)
        self.ctx.bind_pool(self.pool)
        self.workspace = torch.zeros(max(256, self.ctx.workspace_bytes(max_T)), dtype=torch.uint8, device=self.dev)
        if copy_cus is None:
            copy_cus = 16 if S < L * E else 0
        try:
            self._raw_streams = streams_create(copy_cus)
        except Exception:                     # no compute-unit masks on this driver: plain streams
            if copy_cus == 0:
                raise
            copy_cus = 0
            self._raw_streams = streams_create(0)
        self.copy_cus = copy_cus
        self.compute = torch.cuda.ExternalStream(self._raw_streams[0], device=self.dev)
        self.copy = torch.cuda.ExternalStream(self._raw_streams[1], device=self.dev)
        self.host_weights = None
        torch.cuda.synchronize(self.dev)      # the fills above ran on the default stream

    # ---- host weights (pinned)
    def alloc_host_weights(self) -> np.ndarray:
        """Pinned uint16 [L*E, 2*d*F]; returns the numpy view to fill, and binds the blocks."""
        t = torch.empty((self.L * self.E, self.expert_elems), dtype=torch.uint16, pin_memory=True)
        self.host_weights = t
        base, stride = t.data_ptr(), self.expert_bytes
        self.ctx.bind_host_weights([base + i * stride for i in range(self.L * self.E)], keep=t)
        return t.numpy()

    # ---- per-layer tensors
    def to_device(self, x_bits: np.ndarray, ids: np.ndarray, alpha: np.ndarray):
        x = torch.from_numpy(np.ascontiguousarray(x_bits, dtype=np.uint16)).to(self.dev).view(torch.bfloat16)
        i = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to(self.dev)
        a = torch.from_numpy(np.ascontiguousarray(alpha, dtype=np.float32)).to(self.dev)
        y = torch.empty_like(x)
        return x, i, a, y

    def region(self, T, name, dtype, shape):
        """Typed view of one workspace region (see sida_ws_layout)."""
        lay = self.ctx.workspace_layout(T)
        off = getattr(lay, name)
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        return self.workspace[off:off + n].view(dtype).reshape(shape)

    # ---- drive
    def plan_all(self, ids_host_list, layers=None):
        layers = range(len(ids_host_list)) if layers is None else layers
        return [self.ctx.moe_plan(l, np.ascontiguousarray(ids, dtype=np.int32)) for l, ids in zip(layers, ids_host_list)]

    def run(self, plans, xs, idss, alphas, ys):
        self.ctx.run_layers(plans, xs, idss, alphas, ys, self.workspace, self.compute, self.copy)

    # ---- serving loop (Algorithm 1): the hash-building side pushes, the inference side pops and runs
    def push_table(self, tag: int, ids_host: np.ndarray):
        """ids_host: int32 [L, T], the batch's hash table.  Safe to call from another thread."""
        self.ctx.queue_push(tag, np.ascontiguousarray(ids_host, dtype=np.int32))

    def serve_next(self, lookup, timeout_ms=1000):
        """Pops the oldest hash table, plans it and enqueues its L layers.  lookup(tag) returns the
        batch's device tensors (xs, idss, alphas, ys), each a list of L.  Returns (tag, plans), or
        None when no table arrived within the timeout."""
        got = self.ctx.queue_pop_plan(timeout_ms)
        if got is None:
            return None
        tag, _, plans = got
        xs, idss, alphas, ys = lookup(tag)
        self.ctx.run_layers(plans, xs, idss, alphas, ys, self.workspace, self.compute, self.copy)
        return tag, plans

    def sync(self):
        torch.cuda.synchronize(self.dev)      # every stream of the device

    def close(self):
        if self._raw_streams is None:
            return
        self.sync()
        self.ctx.close()
        if self._raw_streams is not None:
            streams_destroy(*self._raw_streams)
            self._raw_streams = None
