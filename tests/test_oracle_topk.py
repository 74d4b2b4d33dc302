"""Pins for the oracle's layer output with k selected experts per token (Eq. 1 of Section 2.1 with
|I| = k; the paper evaluates with the hash function's top-3 experts on two datasets)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from test_oracle_forward import bf16, block
from workloads import bf16_bits_to_f32


def rand_case(rng, T, k, d, F, E):
    x = bf16(rng.standard_normal((T, d)))
    ids = rng.integers(0, E, (T, k)).astype(np.int32)
    alpha = rng.uniform(0.1, 1.0, (T, k)).astype(np.float32)
    blocks = [block(rng.standard_normal((F, d)) * 0.3, rng.standard_normal((d, F)) * 0.3) for _ in range(E)]
    return x, ids, alpha, blocks


def test_hand_computed_integer_case():
    # the two experts of the top-1 hand case; token [1,1] goes to both:
    # expert 0 gives W_out relu(W_in x) = [9, 3], expert 1: pre = [1,1,2] -> [4, -2]
    b0 = block([[1, 2], [-1, 0], [0, 3]], [[1, 0, 2], [0, -1, 1]])
    b1 = block([[0, 1], [2, -1], [1, 1]], [[1, 1, 1], [2, 0, -2]])
    x = bf16([[1, 1], [2, -1]])
    ids = np.array([[0, 1], [1, 1]], dtype=np.int32)
    alpha = np.array([[0.5, 2.0], [1.0, 0.25]], dtype=np.float32)
    y = oracle.moe_forward_topk(x, ids, alpha, [b0, b1], 2, 3)
    # token 0: 0.5*[9,3] + 2*[4,-2] = [12.5, -2.5]
    # token 1 (expert 1 twice): pre = [-1,5,1] -> h = [0,5,1] -> [6,-2]; (1 + 0.25) * [6,-2] = [7.5, -2.5]
    assert y.tolist() == [[12.5, -2.5], [7.5, -2.5]]


def test_k1_is_the_top1_layer():
    rng = np.random.default_rng(11)
    x, ids, alpha, blocks = rand_case(rng, 29, 1, 24, 40, 5)
    a = oracle.moe_forward_topk(x, ids, alpha, blocks, 24, 40)
    b = oracle.moe_forward(x, ids[:, 0], alpha[:, 0], blocks, 24, 40)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_sum_of_k_top1_layers(k):
    rng = np.random.default_rng(12 + k)
    T, d, F, E = 31, 16, 24, 6
    x, ids, alpha, blocks = rand_case(rng, T, k, d, F, E)
    y = oracle.moe_forward_topk(x, ids, alpha, blocks, d, F)
    ref = sum(oracle.moe_forward(x, ids[:, j], alpha[:, j], blocks, d, F).astype(np.float64) for j in range(k))
    np.testing.assert_allclose(y, ref, rtol=2e-6, atol=2e-6 * np.abs(ref).max())


def test_exact_rational_brute_force():
    rng = np.random.default_rng(13)
    T, k, d, F, E = 4, 3, 3, 4, 3
    x = bf16(rng.integers(-4, 5, (T, d)) / 2.0)
    ids = rng.integers(0, E, (T, k)).astype(np.int32)
    alpha = (rng.integers(1, 9, (T, k)) / 8.0).astype(np.float32)
    win = rng.integers(-4, 5, (E, F, d)) / 4.0
    wout = rng.integers(-4, 5, (E, d, F)) / 4.0
    blocks = [block(win[e], wout[e]) for e in range(E)]
    y = oracle.moe_forward_topk(x, ids, alpha, blocks, d, F)
    xf = bf16_bits_to_f32(x)
    for t in range(T):
        for c in range(d):
            acc = Fraction(0)
            for j in range(k):
                e = int(ids[t, j])
                h = [max(Fraction(0), sum(Fraction(float(xf[t, i])) * Fraction(float(win[e, u, i])) for i in range(d)))
                     for u in range(F)]
                acc += Fraction(float(alpha[t, j])) * sum(h[u] * Fraction(float(wout[e, c, u])) for u in range(F))
            assert Fraction(float(y[t, c])) == acc


def test_repeated_expert_adds_the_alphas():
    rng = np.random.default_rng(14)
    T, d, F, E = 17, 16, 24, 4
    x, ids, alpha, blocks = rand_case(rng, T, 2, d, F, E)
    ids[:, 1] = ids[:, 0]
    alpha = (rng.integers(1, 16, (T, 2)) / 16.0).astype(np.float32)       # sums exact in fp32
    y = oracle.moe_forward_topk(x, ids, alpha, blocks, d, F)
    ref = oracle.moe_forward(x, ids[:, 0], alpha.sum(axis=1), blocks, d, F)
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-6 * np.abs(ref).max())


def test_order_of_the_selected_experts_does_not_matter():
    rng = np.random.default_rng(15)
    x, ids, alpha, blocks = rand_case(rng, 13, 3, 16, 24, 5)
    y = oracle.moe_forward_topk(x, ids, alpha, blocks, 16, 24)
    z = oracle.moe_forward_topk(x, ids[:, ::-1], alpha[:, ::-1], blocks, 16, 24)
    np.testing.assert_allclose(y, z, rtol=1e-6, atol=1e-6 * np.abs(y).max())


def test_bad_ids_and_empty():
    rng = np.random.default_rng(16)
    x, ids, alpha, blocks = rand_case(rng, 5, 2, 8, 8, 3)
    bad = ids.copy()
    bad[3, 1] = 3
    with pytest.raises(ValueError):
        oracle.moe_forward_topk(x, bad, alpha, blocks, 8, 8)
    y = oracle.moe_forward_topk(x[:0], ids[:0], alpha[:0], blocks, 8, 8)
    assert y.shape == (0, 8)
