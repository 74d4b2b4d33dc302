"""GPU parity of the hash function (Section 3.4.2) against its float64 oracle: scaling factors
within a tolerance; expert ids as a valid choice (the k most probable experts by the oracle's own
probabilities, up to that tolerance at near-ties); then the predicted table drives a MoE layer."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_18859_amd as sm
from gpu_util import assert_close, bf16_tensor_to_f32, make_runner, say
from oracle import hash_fn
from workloads import Workload, bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu

ALPHA_TOL = 2e-4        # absolute, on probabilities; fp32 network of depth ~ 2 T + 6 against float64


def make_params(rng, d, C, L, E):
    p = {}
    for name, shape in hash_fn.param_shapes(d, C, L, E):
        fan_in = shape[1] if len(shape) == 2 else 1
        scale = 1.5 / np.sqrt(fan_in) if len(shape) == 2 else 0.1
        p[name] = (rng.standard_normal(shape) * scale).astype(np.float32)
    return p


def run_hash(cfg, params, x_bits, n_seq, T):
    dev = torch.device("cuda:0")
    flat = np.concatenate([params[n].reshape(-1) for n, _ in hash_fn.param_shapes(cfg.d_model, cfg.C, cfg.L, cfg.E)])
    assert flat.size == sm.hash_param_count(cfg)
    pd = torch.from_numpy(flat).to(dev)
    xd = torch.from_numpy(x_bits).to(dev)
    N = n_seq * T
    ids = torch.full((cfg.L, N, cfg.top_k), -1, dtype=torch.int32, device=dev)
    alpha = torch.zeros((cfg.L, N, cfg.top_k), dtype=torch.float32, device=dev)
    ws = torch.zeros(sm.hash_workspace_bytes(cfg, N), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    sm.hash_forward(cfg, pd, xd, n_seq, T, ids, alpha, ws, None)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), alpha.cpu().numpy()


@pytest.mark.parametrize("d,C,L,E,k,n_seq,T", [
    (64, 64, 2, 8, 1, 1, 1),
    (64, 64, 3, 5, 2, 2, 17),
    (256, 128, 2, 16, 3, 3, 70),
    (768, 128, 6, 128, 1, 2, 128),
    (768, 128, 6, 128, 3, 1, 200),
    # the dense stages take blocks of 8 tokens from 4096 tokens up and of 2 from 1024 up (ragged last block) ...
    (256, 128, 2, 16, 1, 33, 125),
    (64, 64, 2, 8, 2, 9, 115),
    # ... unless the inputs / logits of a block would not fit the LDS budget: 8 -> 2, 2 -> 1
    (2056, 64, 1, 4, 1, 33, 125),
    (6400, 64, 1, 4, 1, 9, 115),
    (64, 64, 9, 256, 2, 33, 125),
    (64, 64, 30, 256, 1, 9, 115),
])
def test_hash_forward_against_oracle(d, C, L, E, k, n_seq, T):
    say(f"hash function d={d} C={C} L={L} E={E} k={k} sequences={n_seq} x {T}")
    rng = np.random.default_rng(d + C + T)
    cfg = sm.SidaHashConfig(d, C, L, E, k, max(T, 1))
    params = make_params(rng, d, C, L, E)
    x_bits = f32_to_bf16_bits(rng.standard_normal((n_seq * T, d)).astype(np.float32))
    ids, alpha = run_hash(cfg, params, x_bits, n_seq, T)
    x = bf16_bits_to_f32(x_bits)
    worst = 0.0
    for b in range(n_seq):
        want_ids, want_alpha, probs = hash_fn.hash_forward(params, x[b * T:(b + 1) * T], L, E, k)
        got_ids, got_alpha = ids[:, b * T:(b + 1) * T], alpha[:, b * T:(b + 1) * T]
        assert got_ids.min() >= 0 and got_ids.max() < E
        worst = max(worst, float(np.abs(got_alpha - want_alpha).max()))
        for l in range(L):
            for t in range(T):
                chosen = got_ids[l, t].tolist()
                assert len(set(chosen)) == k                                   # k different experts
                # a valid choice: each chosen expert is as probable as the oracle's k-th, up to the tolerance
                assert probs[l, t, chosen].min() >= want_alpha[l, t, k - 1] - ALPHA_TOL
                np.testing.assert_allclose(got_alpha[l, t], probs[l, t, chosen], atol=ALPHA_TOL)
        exact = float((got_ids == want_ids).mean())
        assert exact > 0.97, exact                                             # near-ties are rare
    assert worst <= ALPHA_TOL, worst
    say(f"  max |alpha - oracle| {worst:.2e}")


def test_predicted_table_drives_the_layer():
    """Hash-building side to inference side: the predicted ids / alpha of layer l (top-2) are planned
    and run through the MoE layer, and the result equals the oracle's layer on the same table."""
    d, C, L, E, k, T = 128, 64, 2, 6, 2, 50
    rng = np.random.default_rng(77)
    cfg = sm.SidaHashConfig(d, C, L, E, k, T)
    params = make_params(rng, d, C, L, E)
    x_bits = f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    ids, alpha = run_hash(cfg, params, x_bits, 1, T)
    wl = Workload(500, "hash-to-layer", L, E, d, 256, T * k, None, 4, 2)
    r = make_runner(wl)
    r.ctx.set_top_k(k)
    hw = r.host_weights.numpy()
    for l in range(L):
        plan = r.ctx.moe_plan(l, np.ascontiguousarray(ids[l].reshape(-1)))
        xd, idd, ad, yd = r.to_device(x_bits, ids[l].reshape(-1), alpha[l].reshape(-1))
        r.ctx.moe_layer_forward(plan, xd, idd, ad, yd, r.workspace, r.compute, r.copy)
        r.sync()
        ref = oracle.moe_forward_topk(x_bits, ids[l], alpha[l], [hw[l * E + e] for e in range(E)], d, 256)
        assert_close(bf16_tensor_to_f32(yd), ref, f"layer {l}")
    r.close()


def test_hash_argument_errors():
    dev = torch.device("cuda:0")
    t = torch.zeros(1 << 16, dtype=torch.uint8, device=dev)
    for bad in (sm.SidaHashConfig(64, 96, 1, 4, 1, 8), sm.SidaHashConfig(64, 64, 1, 300, 1, 8),
                sm.SidaHashConfig(64, 64, 1, 4, 5, 8)):
        assert sm.hash_param_count(bad) == 0
        with pytest.raises(sm.SidaError):
            sm.hash_forward(bad, t, t, 1, 4, t, t, t, None)
    assert sm.hash_param_count(sm.SidaHashConfig(68, 64, 1, 4, 1, 8)) == 0          # d_model not a multiple of 8
    ok = sm.SidaHashConfig(64, 64, 1, 4, 1, 8)
    with pytest.raises(sm.SidaError):                     # sequence longer than configured
        sm.hash_forward(ok, t, t, 1, 9, t, t, t, None)
    small = torch.zeros(256, dtype=torch.uint8, device=dev)
    with pytest.raises(sm.SidaError) as e:                # workspace too small
        sm.hash_forward(ok, t, t, 2, 8, t, t, small, None)
    assert e.value.code == -2
