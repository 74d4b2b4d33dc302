"""Shared helpers of the GPU parity tests: build a runner for a workload, run it through the
C ABI, and compare with the oracle."""
import numpy as np
import torch

import oracle
from paper_2310_18859_amd.runner import MoERunner
from workloads import (Workload, bf16_bits_to_f32, fill_host_weights, gen_gate, gen_ids, gen_x)

REL_TOL = 2e-2        # max |y - y_ref| / max |y_ref| per layer, bf16 path vs oracle
ROW_TOL = 2e-2        # the same per token row: max |y[t] - y_ref[t]| / max |y_ref[t]|


def say(*a):
    print(*a, flush=True)


def make_runner(wl: Workload, threads=None) -> MoERunner:
    r = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, wl.S, wl.W, wl.T)
    fill_host_weights(wl, r.alloc_host_weights(), threads=threads)
    return r


def layer_inputs(wl: Workload, layer: int, T=None):
    return gen_x(wl, layer, T), gen_ids(wl, layer, T), gen_gate(wl, layer, T)


def bf16_tensor_to_f32(t: torch.Tensor) -> np.ndarray:
    return bf16_bits_to_f32(t.view(torch.uint16).cpu().numpy())


def oracle_layer(wl: Workload, runner: MoERunner, layer: int, x_bits, ids, alpha, rows=None):
    """Oracle output for the given tokens (optionally only `rows`) of `layer`."""
    hw = runner.host_weights.numpy()
    blocks = [hw[layer * wl.E + e] for e in range(wl.E)]
    if rows is not None:
        x_bits, ids, alpha = x_bits[rows], ids[rows], alpha[rows]
    return oracle.moe_forward(x_bits, ids, alpha, blocks, wl.d_model, wl.d_ff)


def assert_close(y_gpu: np.ndarray, y_ref: np.ndarray, what=""):
    scale = float(np.abs(y_ref).max()) if y_ref.size else 1.0
    if y_ref.size == 0:
        return 0.0
    err = float(np.abs(y_gpu.astype(np.float64) - y_ref).max()) / max(scale, 1e-30)
    l2 = float(np.linalg.norm(y_gpu.astype(np.float64) - y_ref) / max(np.linalg.norm(y_ref), 1e-30))
    assert np.isfinite(y_gpu).all(), what
    assert err <= REL_TOL, f"{what}: max rel err {err:.3e} > {REL_TOL}"
    assert l2 <= 1e-2, f"{what}: rel L2 err {l2:.3e}"
    if y_ref.ndim == 2:                                   # every row against its own largest magnitude
        row_scale = np.abs(y_ref).max(axis=1)
        row_err = np.abs(y_gpu.astype(np.float64) - y_ref).max(axis=1)
        bad = np.nonzero(row_err > ROW_TOL * np.maximum(row_scale, 1e-30))[0]
        assert bad.size == 0, f"{what}: {bad.size} rows off, first {bad[:5]}, worst {float((row_err / np.maximum(row_scale, 1e-30)).max()):.3e}"
    return err
