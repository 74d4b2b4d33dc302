"""Pins for the oracle's layer output (oracle.moe_forward, Eq. 1 with top-1 routing).

Each test compares the oracle with something fixed by mathematics or by a library routine on a
special case, chosen so that a dropped factor, a missing ReLU, a transposed weight matrix or a
wrong expert lookup fails at least one of them."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import bf16_bits_to_f32, f32_to_bf16_bits


def bf16(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def block(w_in, w_out):
    """Pack W_in [F,d] and W_out [d,F] (float) into one bf16 expert block."""
    return np.concatenate([bf16(w_in).reshape(-1), bf16(w_out).reshape(-1)])


def rand_case(rng, T, d, F, E):
    x = bf16(rng.standard_normal((T, d)))
    ids = rng.integers(0, E, T).astype(np.int32)
    alpha = rng.uniform(0.1, 1.0, T).astype(np.float32)
    blocks = [block(rng.standard_normal((F, d)) * 0.3, rng.standard_normal((d, F)) * 0.3) for _ in range(E)]
    return x, ids, alpha, blocks


def test_hand_computed_integer_case():
    # d=2, F=3.  Expert 0: W_in = [[1,2],[-1,0],[0,3]], W_out = [[1,0,2],[0,-1,1]].
    # Expert 1: W_in = [[0,1],[2,-1],[1,1]], W_out = [[1,1,1],[2,0,-2]].
    b0 = block([[1, 2], [-1, 0], [0, 3]], [[1, 0, 2], [0, -1, 1]])
    b1 = block([[0, 1], [2, -1], [1, 1]], [[1, 1, 1], [2, 0, -2]])
    x = bf16([[1, 1], [2, -1], [-1, 2]])
    ids = np.array([0, 1, 0], dtype=np.int32)
    alpha = np.array([0.5, 2.0, 1.0], dtype=np.float32)
    y = oracle.moe_forward(x, ids, alpha, [b0, b1], 2, 3)
    # token 0, expert 0: pre = [3,-1,3] -> h = [3,0,3]; W_out h = [9, 3]; *0.5 = [4.5, 1.5]
    # token 1, expert 1: pre = [-1,5,1] -> h = [0,5,1]; W_out h = [6, -2]; *2 = [12, -4]
    # token 2, expert 0: pre = [3,1,6]  -> h = [3,1,6]; W_out h = [15, 5]; *1 = [15, 5]
    assert y.tolist() == [[4.5, 1.5], [12.0, -4.0], [15.0, 5.0]]


def test_single_expert_equals_dense_ffn_numpy():
    rng = np.random.default_rng(1)
    T, d, F = 37, 48, 80
    x, ids, alpha, blocks = rand_case(rng, T, d, F, 1)
    y = oracle.moe_forward(x, ids, alpha, blocks, d, F)
    xf = bf16_bits_to_f32(x).astype(np.float64)
    w_in = bf16_bits_to_f32(blocks[0][:F * d]).reshape(F, d).astype(np.float64)
    w_out = bf16_bits_to_f32(blocks[0][F * d:]).reshape(d, F).astype(np.float64)
    ref = (np.maximum(xf @ w_in.T, 0.0) @ w_out.T) * alpha.astype(np.float64)[:, None]
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-6 * np.abs(ref).max())


def test_exact_rational_brute_force_tiny():
    rng = np.random.default_rng(2)
    T, d, F, E = 6, 3, 5, 3
    x, ids, alpha, blocks = rand_case(rng, T, d, F, E)
    y = oracle.moe_forward(x, ids, alpha, blocks, d, F)
    xf = bf16_bits_to_f32(x)
    for t in range(T):
        w = bf16_bits_to_f32(blocks[ids[t]])
        w_in = [[Fraction(float(w[j * d + i])) for i in range(d)] for j in range(F)]
        w_out = [[Fraction(float(w[F * d + c * F + j])) for j in range(F)] for c in range(d)]
        xt = [Fraction(float(v)) for v in xf[t]]
        h = [max(Fraction(0), sum(w_in[j][i] * xt[i] for i in range(d))) for j in range(F)]
        for c in range(d):
            exact = Fraction(float(alpha[t])) * sum(w_out[c][j] * h[j] for j in range(F))
            assert abs(float(exact) - float(y[t, c])) <= 1e-6 * max(1.0, abs(float(exact)))


def test_rank_one_closed_form_catches_transposes():
    # W_in[j,i] = a_j b_i and W_out[c,j] = u_c v_j  =>  y_c = alpha u_c sum_j v_j relu(a_j (b.x))
    rng = np.random.default_rng(3)
    T, d, F = 9, 4, 7
    a = bf16_bits_to_f32(bf16(rng.integers(-3, 4, F))).astype(np.float64)
    b = bf16_bits_to_f32(bf16(rng.integers(-3, 4, d))).astype(np.float64)
    u = bf16_bits_to_f32(bf16(rng.integers(-3, 4, d))).astype(np.float64)
    v = bf16_bits_to_f32(bf16(rng.integers(-3, 4, F))).astype(np.float64)
    x = bf16(rng.integers(-4, 5, (T, d)))
    alpha = rng.uniform(0.1, 1.0, T).astype(np.float32)
    ids = np.zeros(T, dtype=np.int32)
    y = oracle.moe_forward(x, ids, alpha, [block(np.outer(a, b), np.outer(u, v))], d, F)
    s = bf16_bits_to_f32(x).astype(np.float64) @ b
    inner = (np.maximum(np.outer(s, a), 0.0) * v).sum(axis=1)
    ref = alpha.astype(np.float64)[:, None] * inner[:, None] * u[None, :]
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-9)


def test_identity_experts_unit_gates_return_x():
    rng = np.random.default_rng(4)
    T, d, E = 33, 16, 4
    x = bf16(np.abs(rng.standard_normal((T, d))))
    ids = rng.integers(0, E, T).astype(np.int32)
    eye = np.eye(d)
    y = oracle.moe_forward(x, ids, np.ones(T, np.float32), [block(eye, eye)] * E, d, d)
    assert np.array_equal(y, bf16_bits_to_f32(x))


def test_relu_zeroes_negative_preactivations():
    rng = np.random.default_rng(5)
    T, d = 8, 6
    x = bf16(np.abs(rng.standard_normal((T, d))) + 0.5)
    y = oracle.moe_forward(x, np.zeros(T, np.int32), np.ones(T, np.float32),
                           [block(-np.eye(d), np.eye(d))], d, d)
    assert np.all(y == 0.0)


def test_each_token_uses_its_own_expert_and_gate():
    rng = np.random.default_rng(6)
    T, d, E = 40, 8, 5
    scale = [1.0, 2.0, 4.0, 0.5, 8.0]
    x = bf16(np.abs(rng.standard_normal((T, d))))
    ids = rng.integers(0, E, T).astype(np.int32)
    alpha = (2.0 ** rng.integers(-3, 3, T)).astype(np.float32)
    blocks = [block(np.eye(d), scale[e] * np.eye(d)) for e in range(E)]
    y = oracle.moe_forward(x, ids, alpha, blocks, d, d)
    ref = bf16_bits_to_f32(x) * (alpha * np.array(scale, np.float32)[ids])[:, None]
    assert np.array_equal(y, ref)


def test_permutation_equivariance_and_token_independence():
    rng = np.random.default_rng(7)
    T, d, F, E = 50, 12, 20, 6
    x, ids, alpha, blocks = rand_case(rng, T, d, F, E)
    y = oracle.moe_forward(x, ids, alpha, blocks, d, F)
    p = rng.permutation(T)
    yp = oracle.moe_forward(x[p], ids[p], alpha[p], blocks, d, F)
    assert np.array_equal(yp, y[p])
    keep = np.sort(rng.choice(T, 11, replace=False))
    yk = oracle.moe_forward(x[keep], ids[keep], alpha[keep], blocks, d, F)
    assert np.array_equal(yk, y[keep])


def test_linear_in_alpha():
    rng = np.random.default_rng(8)
    T, d, F, E = 20, 8, 24, 3
    x, ids, alpha, blocks = rand_case(rng, T, d, F, E)
    y1 = oracle.moe_forward(x, ids, np.ones(T, np.float32), blocks, d, F)
    y4 = oracle.moe_forward(x, ids, np.full(T, 4.0, np.float32), blocks, d, F)
    assert np.array_equal(y4, 4.0 * y1)           # scaling by a power of two is exact


def test_bad_id_rejected():
    rng = np.random.default_rng(9)
    x, ids, alpha, blocks = rand_case(rng, 4, 4, 4, 2)
    ids[2] = 2
    with pytest.raises(ValueError):
        oracle.moe_forward(x, ids, alpha, blocks, 4, 4)
    ids[2] = -1
    with pytest.raises(ValueError):
        oracle.moe_forward(x, ids, alpha, blocks, 4, 4)


def test_empty_batch():
    rng = np.random.default_rng(10)
    _, _, _, blocks = rand_case(rng, 1, 4, 4, 2)
    y = oracle.moe_forward(np.zeros((0, 4), np.uint16), np.zeros(0, np.int32), np.zeros(0, np.float32), blocks, 4, 4)
    assert y.shape == (0, 4)
