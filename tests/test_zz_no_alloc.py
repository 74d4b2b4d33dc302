"""The entry point that allocates nothing (sida_hash_forward_static): its scratch is a static
device array inside the library.  Checked through the C ABI against sida_hash_forward (same
kernels, caller's workspace) on two calls in a row, the second with a smaller input, so stale
contents of the shared array would show."""
import numpy as np
import pytest
import torch

import paper_2310_18859_amd as sm
from gpu_util import say
from oracle import hash_fn
from test_gpu_hash import make_params
from workloads import f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def both(cfg, flat_params, x_bits, n_seq, T):
    dev = torch.device("cuda:0")
    pd = torch.from_numpy(flat_params).to(dev)
    xd = torch.from_numpy(x_bits).to(dev)
    N = n_seq * T
    out = []
    for static in (False, True):
        ids = torch.full((cfg.L, N, cfg.top_k), -1, dtype=torch.int32, device=dev)
        alpha = torch.full((cfg.L, N, cfg.top_k), -1.0, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        if static:
            sm.hash_forward_static(cfg, pd, xd, n_seq, T, ids, alpha, None)
        else:
            ws = torch.zeros(sm.hash_workspace_bytes(cfg, N), dtype=torch.uint8, device=dev)
            sm.hash_forward(cfg, pd, xd, n_seq, T, ids, alpha, ws, None)
        torch.cuda.synchronize()
        out.append((ids.cpu().numpy(), alpha.cpu().numpy()))
    return out


def test_static_scratch_equals_workspace_variant_on_two_calls_in_a_row():
    d, C, L, E, k = 256, 128, 3, 16, 2
    rng = np.random.default_rng(5)
    params = make_params(rng, d, C, L, E)
    flat = np.concatenate([params[n].reshape(-1) for n, _ in hash_fn.param_shapes(d, C, L, E)])
    for n_seq, T in ((9, 130), (2, 37)):                     # the second call is smaller than the first
        say(f"no-allocation hash forward: {n_seq} sequences x {T} tokens")
        cfg = sm.SidaHashConfig(d, C, L, E, k, 256)
        x_bits = f32_to_bf16_bits(rng.standard_normal((n_seq * T, d)).astype(np.float32))
        (ids_a, alpha_a), (ids_b, alpha_b) = both(cfg, flat, x_bits, n_seq, T)
        assert ids_a.min() >= 0 and alpha_a.min() > 0
        assert np.array_equal(ids_a, ids_b)                   # same kernels, same inputs: identical
        assert np.array_equal(alpha_a, alpha_b)


def test_static_scratch_rejects_what_does_not_fit():
    dev = torch.device("cuda:0")
    cfg = sm.SidaHashConfig(64, 128, 1, 4, 1, 4096)
    t = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    assert sm.hash_workspace_bytes(cfg, 4096) > (16 << 20) >= sm.hash_workspace_bytes(cfg, 4095)
    with pytest.raises(sm.SidaError) as e:
        sm.hash_forward_static(cfg, t, t, 1, 4096, t, t, None)
    assert e.value.code == -2
    with pytest.raises(sm.SidaError) as e:                    # a bad config is still an argument error
        sm.hash_forward_static(sm.SidaHashConfig(64, 96, 1, 4, 1, 8), t, t, 1, 4, t, t, None)
    assert e.value.code == -1
