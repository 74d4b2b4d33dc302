"""GPU parity of the single stages, through the C ABI: counting sort / gather (bit-exact) and
gate-weighted combine."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bf16_tensor_to_f32, say
from paper_2310_18859_amd.runner import MoERunner
from workloads import bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def ids_for(rng, kind, T, E):
    if kind == "uniform":
        return rng.integers(0, E, T).astype(np.int32)
    if kind == "zipf":
        return np.minimum(rng.zipf(1.3, T) - 1, E - 1).astype(np.int32)
    if kind == "one":
        return np.full(T, E - 1, dtype=np.int32)
    raise ValueError(kind)


@pytest.mark.parametrize("T,E,kind", [
    (1, 1, "one"), (1, 8, "uniform"), (63, 8, "uniform"), (64, 8, "zipf"), (65, 3, "uniform"),
    (255, 64, "zipf"), (256, 256, "uniform"), (257, 256, "zipf"), (1000, 7, "one"), (1023, 128, "zipf"),
    (2047, 200, "zipf"), (2048, 128, "uniform"), (2049, 128, "zipf"),    # around the single-workgroup sort's limit
    (4095, 128, "zipf"), (4096, 256, "uniform"), (5000, 256, "uniform"), (4097, 64, "zipf"),
    (8191, 128, "zipf"), (8192, 256, "zipf"), (8193, 128, "uniform"),                    # ... and its larger shapes
    (16384, 128, "zipf"), (32768, 256, "zipf"),
    (65536, 128, "uniform"), (65537, 256, "zipf"), (70001, 64, "zipf"),
])
def test_dispatch_bit_exact(T, E, kind):
    say(f"dispatch T={T} E={E} {kind}")
    rng = np.random.default_rng(T * 1000 + E)
    d = 128
    r = MoERunner(1, E, d, 128, 1, 1, T)
    ids = ids_for(rng, kind, T, E)
    x_bits = rng.integers(0, 2 ** 16, (T, d)).astype(np.uint16)       # any bit pattern must survive the move
    x, i, a, y = r.to_device(x_bits, ids, np.ones(T, np.float32))
    r.workspace.fill_(0xEE)
    r.sync()
    r.ctx.dispatch(x, i, T, r.workspace, r.compute)
    r.sync()
    counts, offsets = oracle.token_counts(ids, E)
    if T * E <= 300000:
        perm, inv = oracle.stable_order(ids, E)
    else:        # the plain double loop is slow here; numpy's stable argsort is what the oracle is pinned to
        perm = np.argsort(ids, kind="stable").astype(np.int32)
        inv = np.empty(T, np.int32)
        inv[perm] = np.arange(T, dtype=np.int32)
    assert np.array_equal(r.region(T, "counts", torch.int32, (E,)).cpu().numpy(), counts)
    assert np.array_equal(r.region(T, "offsets", torch.int32, (E + 1,)).cpu().numpy(), offsets)
    assert np.array_equal(r.region(T, "perm", torch.int32, (T,)).cpu().numpy(), perm)
    assert np.array_equal(r.region(T, "inv", torch.int32, (T,)).cpu().numpy(), inv)
    xp = r.region(T, "x_perm", torch.uint16, (T, d)).cpu().numpy()
    assert np.array_equal(xp, oracle.dispatch(x_bits, perm))
    r.close()


@pytest.mark.parametrize("T,d", [(1, 128), (77, 128), (300, 768), (1025, 1024)])
def test_combine(T, d):
    say(f"combine T={T} d={d}")
    rng = np.random.default_rng(T + d)
    r = MoERunner(1, 4, d, 128, 1, 1, T)
    yp_bits = f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    inv = rng.permutation(T).astype(np.int32)
    alpha = rng.uniform(0.1, 1.0, T).astype(np.float32)
    r.region(T, "y_perm", torch.uint16, (T, d)).copy_(torch.from_numpy(yp_bits))
    r.region(T, "inv", torch.int32, (T,)).copy_(torch.from_numpy(inv))
    a = torch.from_numpy(alpha).to(r.dev)
    y = torch.empty((T, d), dtype=torch.bfloat16, device=r.dev)
    r.ctx.combine(a, T, y, r.workspace, r.compute)
    r.sync()
    got = y.view(torch.uint16).cpu().numpy()
    yp = bf16_bits_to_f32(yp_bits)
    ref64 = oracle.combine(yp, inv, alpha)
    # same decision precision as the kernel: fp32 product, one round-to-nearest-even to bf16
    want = f32_to_bf16_bits(alpha[:, None] * yp[inv])
    assert np.array_equal(got, want)
    np.testing.assert_allclose(bf16_bits_to_f32(got), ref64, rtol=2 ** -8, atol=0)
    r.close()


def test_dispatch_then_combine_is_identity_on_gpu():
    say("dispatch->combine identity")
    T, d, E = 3001, 768, 64
    rng = np.random.default_rng(5)
    r = MoERunner(1, E, d, 128, 1, 1, T)
    x_bits = f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    ids = ids_for(rng, "zipf", T, E)
    x, i, a, y = r.to_device(x_bits, ids, np.ones(T, np.float32))
    r.ctx.dispatch(x, i, T, r.workspace, r.compute)
    with torch.cuda.stream(r.compute):                 # identity experts: y_perm := x_perm
        r.region(T, "y_perm", torch.uint16, (T, d)).copy_(r.region(T, "x_perm", torch.uint16, (T, d)))
    r.ctx.combine(a, T, y, r.workspace, r.compute)
    r.sync()
    assert np.array_equal(y.view(torch.uint16).cpu().numpy(), x_bits)
    r.close()
