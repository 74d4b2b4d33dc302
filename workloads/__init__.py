"""Seeded synthetic inputs for the SiDA-MoE layer hot path.

This module only *draws inputs*: token activations, expert ids, gate values and
expert weights with the shapes of Switch-base / Switch-large MoE layers.  It holds
none of the method's arithmetic (no sorting, planning, FFN or combine) and is the
only module shared by the CPU oracle's tests and the HIP path's tests / benchmark.

The paper evaluates on SST2 / MRPC / MultiRC sentences fed to Switch Transformers
(Section 4, "Setup"); none of those are reproduced here.  The arrays below stand in
for them: only the layer dimensions and a skewed (Zipf) expert popularity, in the
spirit of the sentence-level activation sparsity of Section 2.4, are kept.

Every array is drawn from its own ``numpy`` PCG64 stream keyed by
``SeedSequence([20231018, cfg, layer, stream])`` so any piece can be regenerated
on its own (stream 0: x, 1: ids, 2: gate, 3: expert permutation, 4+e: weights of
expert e).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20231018

STREAM_X, STREAM_IDS, STREAM_GATE, STREAM_PERM, STREAM_W0 = 0, 1, 2, 3, 4
STREAM_BATCH_IDS = 1000   # ids of batch b of a stream: seed sequence [base, cfg, layer, 1000, b]


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: L MoE layers of E experts, T tokens per layer.

    ``S`` is the number of expert slots of the HBM pool, ``W`` the largest number of
    experts computed together as one wave (W <= S).  ``zipf_s`` is None for uniform ids.
    """
    index: int
    name: str
    L: int
    E: int
    d_model: int
    d_ff: int
    T: int
    zipf_s: float | None
    S: int
    W: int

    @property
    def expert_elems(self) -> int:
        return 2 * self.d_model * self.d_ff

    @property
    def expert_bytes(self) -> int:
        return 2 * self.expert_elems

    def scaled(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


def _w(S: int, n_active_hint: int) -> int:
    # all activated experts fit: one wave may hold them all; otherwise half the pool,
    # so the copy of the next wave can overlap the compute of the current one.
    return S if n_active_hint <= S else max(1, S // 2)


WORKLOADS = (
    Workload(0, "switch-8-T256", 1, 8, 768, 3072, 256, None, 8, 8),
    Workload(1, "switch-base-64-T8192", 6, 64, 768, 3072, 8192, 1.2, 6 * 64, 64),
    Workload(2, "switch-base-128-T16384", 6, 128, 768, 3072, 16384, 1.0, 32, _w(32, 128)),
    Workload(3, "switch-base-256-T32768", 6, 256, 768, 3072, 32768, 0.8, 48, _w(48, 256)),
    Workload(4, "switch-large-128-T32768", 12, 128, 1024, 4096, 32768, 1.2, 64, _w(64, 128)),
)


def rng_for(cfg: int, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, cfg, layer, stream])))


# ----------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns.

    Inputs here are finite, so no NaN handling is needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- per-array draws
def gen_x(wl: Workload, layer: int, T: int | None = None) -> np.ndarray:
    """Token activations of one layer: N(0,1), rounded to bf16.  uint16 [T, d_model]."""
    T = wl.T if T is None else T
    g = rng_for(wl.index, layer, STREAM_X)
    return f32_to_bf16_bits(g.standard_normal((T, wl.d_model), dtype=np.float32))


def gen_gate(wl: Workload, layer: int, T: int | None = None) -> np.ndarray:
    """Per-token scaling factor alpha: U(0.1, 1), float32 [T]."""
    T = wl.T if T is None else T
    g = rng_for(wl.index, layer, STREAM_GATE)
    return g.uniform(0.1, 1.0, T).astype(np.float32)


def expert_permutation(wl: Workload, layer: int) -> np.ndarray:
    g = rng_for(wl.index, layer, STREAM_PERM)
    return g.permutation(wl.E).astype(np.int32)


def gen_ids(wl: Workload, layer: int, T: int | None = None) -> np.ndarray:
    """Predicted expert id per token, int32 [T].

    Uniform over the experts when ``zipf_s`` is None; otherwise popularity rank k=1..E is
    drawn with probability proportional to k**(-s) and mapped through a seeded permutation
    of the experts, so the popular experts differ from layer to layer."""
    T = wl.T if T is None else T
    g = rng_for(wl.index, layer, STREAM_IDS)
    if wl.zipf_s is None:
        return g.integers(0, wl.E, T).astype(np.int32)
    p = np.arange(1, wl.E + 1, dtype=np.float64) ** (-float(wl.zipf_s))
    cdf = np.cumsum(p / p.sum())
    rank = np.searchsorted(cdf, g.random(T), side="right")
    rank = np.minimum(rank, wl.E - 1)
    return expert_permutation(wl, layer)[rank].astype(np.int32)


def gen_batch_ids(wl: Workload, batch: int, T: int) -> np.ndarray:
    """Hash table of one batch of a stream (Section 3.1): predicted expert ids of T tokens for every
    MoE layer, int32 [L, T].  Same popularity law and per-layer expert permutation as ``gen_ids`` -
    so the experts that are popular in one batch are popular in the next, which is what makes a
    slot pool hit across batches - with an independent draw per (batch, layer).  With T around 100
    and Zipf(1.0) over 128 experts a batch activates about 35-40 % of a layer's experts, the
    sentence-level sparsity Section 2.4 reports for Switch-base-128."""
    out = np.empty((wl.L, T), dtype=np.int32)
    for layer in range(wl.L):
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(
            [BASE_SEED, wl.index, layer, STREAM_BATCH_IDS, batch])))
        if wl.zipf_s is None:
            out[layer] = g.integers(0, wl.E, T)
            continue
        p = np.arange(1, wl.E + 1, dtype=np.float64) ** (-float(wl.zipf_s))
        cdf = np.cumsum(p / p.sum())
        rank = np.minimum(np.searchsorted(cdf, g.random(T), side="right"), wl.E - 1)
        out[layer] = expert_permutation(wl, layer)[rank]
    return out


def gen_expert_block(wl: Workload, layer: int, e: int, out: np.ndarray | None = None) -> np.ndarray:
    """Weights of one expert as one contiguous bf16 block, uint16 [2*d*F]:
    first W_in as [d_ff, d_model] (row j = the weights of hidden unit j), then
    W_out as [d_model, d_ff].  Values are 0.02 * N(0,1), rounded to bf16."""
    g = rng_for(wl.index, layer, STREAM_W0 + e)
    w = g.standard_normal(wl.expert_elems, dtype=np.float32)
    w *= np.float32(0.02)
    bits = f32_to_bf16_bits(w)
    if out is None:
        return bits
    out[...] = bits
    return out


def fill_host_weights(wl: Workload, out: np.ndarray, threads: int | None = None,
                      progress=None) -> np.ndarray:
    """Fill ``out`` (uint16 [L*E, 2*d*F], e.g. a view of pinned memory) with every expert's block.
    Rows are keyed ``layer*E + e``.  Uses a thread pool: numpy releases the GIL in the draws."""
    assert out.shape == (wl.L * wl.E, wl.expert_elems) and out.dtype == np.uint16
    threads = threads or min(16, os.cpu_count() or 1)
    keys = [(l, e) for l in range(wl.L) for e in range(wl.E)]

    def one(k):
        l, e = k
        gen_expert_block(wl, l, e, out[l * wl.E + e])
        return k

    with ThreadPoolExecutor(threads) as ex:
        for i, _ in enumerate(ex.map(one, keys)):
            if progress is not None and (i + 1) % 128 == 0:
                progress(i + 1, len(keys))
    return out
