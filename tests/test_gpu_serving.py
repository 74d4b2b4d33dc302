"""GPU parity of the serving loop: a stream of batches goes through the hash-table queue, the
slot pool persists across batches (Section 3.1), every batch's outputs must equal the oracle's
and the plans the oracle's serving loop, for each replacement policy."""
import threading

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, bf16_tensor_to_f32, make_runner, oracle_layer, say
from test_abi_host import plans_equal
from workloads import WORKLOADS, gen_batch_ids, gen_gate, gen_x

pytestmark = pytest.mark.gpu


def stream(wl, n_batches, T):
    tables = [gen_batch_ids(wl, b, T) for b in range(n_batches)]
    xs = [[gen_x(wl.scaled(index=wl.index + 100 + b), l, T) for l in range(wl.L)] for b in range(n_batches)]
    gates = [[gen_gate(wl.scaled(index=wl.index + 100 + b), l, T) for l in range(wl.L)] for b in range(n_batches)]
    return tables, xs, gates


@pytest.mark.parametrize("policy,look", [("fifo", 0), ("lru", 0), ("belady", 2)])
def test_stream_of_batches_small(policy, look):
    wl = WORKLOADS[0].scaled(L=3, E=12, d_model=128, d_ff=256, T=48, zipf_s=1.1, S=30, W=4, name="serve-small")
    n = 7
    tables, xs, gates = stream(wl, n, wl.T)
    r = make_runner(wl)
    r.ctx.set_policy(policy, look)
    dev = {b: tuple(zip(*[r.to_device(xs[b][l], tables[b][l], gates[b][l]) for l in range(wl.L)])) for b in range(n)}
    r.sync()
    for b in range(n):                                  # the whole stream is queued first: fixed look-ahead
        r.push_table(b, tables[b])
    want = oracle.serve_plans(oracle.PoolState(wl.E, wl.S, policy), [t.tolist() for t in tables], wl.W, look)
    loads = 0
    for b in range(n):
        say(f"[serve {policy}] batch {b}")
        tag, plans = r.serve_next(lambda t: [list(v) for v in dev[t]], 0)
        assert tag == b
        for p, q in zip(plans, want[b]):
            plans_equal(p, q, wl.E)
        loads += sum(p.n_miss for p in plans)
    assert r.serve_next(lambda t: None, 0) is None
    r.sync()
    active = sum(len(set(t[l].tolist())) for t in tables for l in range(wl.L))
    say(f"[serve {policy}] {loads} loads for {active} activations")
    assert loads < active                               # later batches hit experts loaded by earlier ones
    for b in range(n):
        for l in range(wl.L):
            y = bf16_tensor_to_f32(dev[b][3][l])
            assert_close(y, oracle_layer(wl, r, l, xs[b][l], tables[b][l], gates[b][l]), f"batch {b} layer {l}")
    r.close()


def test_two_threads_sentence_sized_batches():
    """Switch-base-128 layer shape, 128-token batches, a producer thread pushing hash tables while
    the inference side pops and runs; outputs of sampled rows against the oracle."""
    wl = WORKLOADS[2].scaled(L=2, T=128, S=96, W=48, name="serve-base128")
    n = 6
    tables, xs, gates = stream(wl, n, wl.T)
    r = make_runner(wl)
    r.ctx.set_policy("belady", 3)
    dev = {b: tuple(zip(*[r.to_device(xs[b][l], tables[b][l], gates[b][l]) for l in range(wl.L)])) for b in range(n)}
    r.sync()

    def producer():
        for b in range(n):
            r.push_table(b, tables[b])
        r.ctx.queue_close()

    th = threading.Thread(target=producer)
    th.start()
    served, loads, active = [], 0, 0
    while True:
        try:
            got = r.serve_next(lambda t: [list(v) for v in dev[t]], 2000)
        except Exception as e:                          # closed and drained
            assert getattr(e, "code", None) == -7
            break
        assert got is not None
        served.append(got[0])
        loads += sum(p.n_miss for p in got[1])
        active += sum(p.n_active for p in got[1])
        for p in got[1]:                                # whatever the look-ahead was, a plan is consistent
            assert p.n_waves >= 1 and sum(list(p.counts)[:wl.E]) == wl.T
    th.join()
    r.sync()
    assert served == list(range(n)) and loads < active
    say(f"[serve threads] {loads} loads for {active} activations")
    rows = np.arange(0, wl.T, 5)
    for b in range(n):
        for l in range(wl.L):
            y = bf16_tensor_to_f32(dev[b][3][l])[rows]
            assert_close(y, oracle_layer(wl, r, l, xs[b][l], tables[b][l], gates[b][l], rows), f"batch {b} layer {l}")
    r.close()


def test_hash_thread_feeds_inference_thread():
    """Algorithm 1 with both of its threads: the hash-building thread runs the hash function on the
    GPU (its own stream), copies the predicted ids to the host and queues them; the inference
    thread pops, plans and runs the MoE layers with the predicted ids and scaling factors."""
    import paper_2310_18859_amd as sm
    from oracle import hash_fn
    from test_gpu_hash import make_params
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits

    d, C, L, E, T, n = 128, 64, 2, 10, 40, 5
    wl = WORKLOADS[0].scaled(L=L, E=E, d_model=d, d_ff=256, T=T, S=8, W=4, name="serve-hash")
    rng = np.random.default_rng(11)
    cfg = sm.SidaHashConfig(d, C, L, E, 1, T)
    params = make_params(rng, d, C, L, E)
    r = make_runner(wl)
    r.ctx.set_policy("belady", 2)
    dev = r.dev
    flat = np.concatenate([params[nm].reshape(-1) for nm, _ in hash_fn.param_shapes(d, C, L, E)])
    pd = torch.from_numpy(flat).to(dev)
    x_bits = [f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32)) for _ in range(n)]
    xd = [torch.from_numpy(b).to(dev) for b in x_bits]
    ids_d = [torch.zeros((L, T, 1), dtype=torch.int32, device=dev) for _ in range(n)]
    alpha_d = [torch.zeros((L, T, 1), dtype=torch.float32, device=dev) for _ in range(n)]
    ys = [[torch.zeros((T, d), dtype=torch.bfloat16, device=dev) for _ in range(L)] for _ in range(n)]
    ws = torch.zeros(sm.hash_workspace_bytes(cfg, T), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    hash_stream = torch.cuda.Stream(device=dev)
    tables = [None] * n

    def hash_thread():
        for b in range(n):
            sm.hash_forward(cfg, pd, xd[b], 1, T, ids_d[b], alpha_d[b], ws, hash_stream)
            hash_stream.synchronize()                     # the table must be complete before it is queued
            tables[b] = ids_d[b].cpu().numpy().reshape(L, T)
            r.push_table(b, tables[b])
        r.ctx.queue_close()

    th = threading.Thread(target=hash_thread)
    th.start()
    served = 0
    while True:
        try:
            got = r.serve_next(lambda t: ([xd[t].view(torch.bfloat16)] * L, [ids_d[t][l].reshape(-1) for l in range(L)],
                                          [alpha_d[t][l].reshape(-1) for l in range(L)], ys[t]), 5000)
        except sm.SidaError as e:
            assert e.code == -7
            break
        assert got is not None and got[0] == served
        served += 1
    th.join()
    r.sync()
    assert served == n
    hw = r.host_weights.numpy()
    for b in range(n):
        alpha = alpha_d[b].cpu().numpy().reshape(L, T)
        for l in range(L):
            ref = oracle.moe_forward(x_bits[b], tables[b][l], alpha[l], [hw[l * E + e] for e in range(E)], d, 256)
            assert_close(bf16_tensor_to_f32(ys[b][l]), ref, f"batch {b} layer {l}")
    r.close()
