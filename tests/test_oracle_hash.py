"""Pins for the oracle of the hash function (Section 3.4.2): SparseMax, the LSTM, the whole forward."""
import itertools

import numpy as np
import pytest
import torch

from oracle import hash_fn


def project_by_exhaustive_search(z):
    """The simplex projection found by trying every support set: on support S the solution is
    z_i - tau with tau = (sum_S z - 1) / |S|; the right S is the one whose solution is feasible
    (positive on S) and satisfies the optimality condition z_j <= tau off S."""
    n = len(z)
    for size in range(1, n + 1):
        for S in itertools.combinations(range(n), size):
            tau = (sum(z[i] for i in S) - 1.0) / size
            if all(z[i] - tau > 0 for i in S) and all(z[j] <= tau + 1e-15 for j in range(n) if j not in S):
                p = np.zeros(n)
                for i in S:
                    p[i] = z[i] - tau
                return p
    raise AssertionError("no support found")


@pytest.mark.parametrize("seed", range(30))
def test_sparsemax_equals_exhaustive_projection(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 8))
    z = rng.standard_normal(n) * rng.choice([0.3, 1.0, 4.0])
    np.testing.assert_allclose(hash_fn.sparsemax(z), project_by_exhaustive_search(z), atol=1e-12)


def test_sparsemax_known_values_and_properties():
    assert hash_fn.sparsemax([0.3, 0.3]).tolist() == [0.5, 0.5]
    assert hash_fn.sparsemax([2.0, 0.0, -1.0]).tolist() == [1.0, 0.0, 0.0]        # a gap of >= 1 is one-hot
    np.testing.assert_allclose(hash_fn.sparsemax([0.6, 0.4, -3.0]), [0.6, 0.4, 0.0], atol=1e-15)
    rng = np.random.default_rng(3)
    for _ in range(50):
        z = rng.standard_normal(int(rng.integers(2, 40))) * 2
        p = hash_fn.sparsemax(z)
        assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
        np.testing.assert_allclose(hash_fn.sparsemax(z + 7.5), p, atol=1e-12)     # shift invariance
        assert (np.argsort(-p, kind="stable")[:1] == np.argsort(-z, kind="stable")[:1]).all()
        # the projection is the closest point of the simplex: no random feasible point is closer
        for _ in range(20):
            q = rng.dirichlet(np.ones(len(z)))
            assert np.sum((p - z) ** 2) <= np.sum((q - z) ** 2) + 1e-12


@pytest.mark.parametrize("T,I,H", [(1, 3, 2), (7, 5, 4), (23, 16, 16)])
def test_lstm_equals_torch(T, I, H):
    rng = np.random.default_rng(T + I)
    ref = torch.nn.LSTM(I, H, num_layers=2, batch_first=True).double()
    x = rng.standard_normal((T, I))
    with torch.no_grad():
        want = ref(torch.from_numpy(x)[None])[0][0].numpy()
    g = lambda n: getattr(ref, n).detach().numpy()
    h1 = hash_fn.lstm_layer(x, g("weight_ih_l0"), g("weight_hh_l0"), g("bias_ih_l0"), g("bias_hh_l0"))
    h2 = hash_fn.lstm_layer(h1, g("weight_ih_l1"), g("weight_hh_l1"), g("bias_ih_l1"), g("bias_hh_l1"))
    np.testing.assert_allclose(h2, want, rtol=1e-10, atol=1e-12)


def random_params(rng, d, C, L, E, scale=0.3):
    return {n: rng.standard_normal(s) * scale for n, s in hash_fn.param_shapes(d, C, L, E)}


def test_forward_shapes_and_probabilities():
    rng = np.random.default_rng(1)
    d, C, L, E, k, T = 12, 8, 3, 5, 2, 9
    ids, alpha, probs = hash_fn.hash_forward(random_params(rng, d, C, L, E), rng.standard_normal((T, d)), L, E, k)
    assert ids.shape == (L, T, k) and alpha.shape == (L, T, k) and probs.shape == (L, T, E)
    np.testing.assert_allclose(probs.sum(axis=2), 1.0, atol=1e-12)
    for l in range(L):
        for t in range(T):
            want = np.argsort(-probs[l, t], kind="stable")[:k]
            assert ids[l, t].tolist() == want.tolist()
            np.testing.assert_allclose(alpha[l, t], probs[l, t, want])
            assert alpha[l, t, 0] >= alpha[l, t, 1]


def test_forward_with_silent_sequence_model_is_a_linear_classifier():
    """With the LSTM's output gates shut (large negative output-gate bias) its output is ~0, every
    attention row is uniform over zeros, and the prediction reduces to
    softmax(W_out (W_in x + b_in) + b_out): the residual path alone."""
    rng = np.random.default_rng(2)
    d, C, L, E, T = 6, 4, 2, 7, 5
    p = random_params(rng, d, C, L, E)
    for n in ("b_ih1", "b_ih2"):
        p[n][3 * C:] = -60.0
    x = rng.standard_normal((T, d))
    ids, alpha, probs = hash_fn.hash_forward(p, x, L, E, 1)
    z = (x @ p["w_in"].T + p["b_in"]) @ p["w_out"].T + p["b_out"]
    for l in range(L):
        zl = z[:, l * E:(l + 1) * E]
        want = np.exp(zl) / np.exp(zl).sum(axis=1, keepdims=True)
        np.testing.assert_allclose(probs[l], want, atol=1e-10)
        assert ids[l, :, 0].tolist() == want.argmax(axis=1).tolist()


def test_attention_on_a_one_token_sequence_returns_the_token():
    rng = np.random.default_rng(4)
    d, C, L, E = 5, 4, 1, 3
    p = random_params(rng, d, C, L, E)
    x = rng.standard_normal((1, d))
    _, _, probs = hash_fn.hash_forward(p, x, L, E, 1)
    c0 = x @ p["w_in"].T + p["b_in"]
    h1 = hash_fn.lstm_layer(c0, p["w_ih1"], p["w_hh1"], p["b_ih1"], p["b_hh1"])
    h2 = hash_fn.lstm_layer(h1, p["w_ih2"], p["w_hh2"], p["b_ih2"], p["b_hh2"])
    z = (h2 + c0) @ p["w_out"].T + p["b_out"]                             # sparsemax of one score is [1]
    np.testing.assert_allclose(probs[0], np.exp(z) / np.exp(z).sum(), atol=1e-12)


# ---- the attention layer on sequences of more than one token -------------------------------------
def test_attention_hand_worked_sequences():
    from golden_io import read_attention_cases
    cases = read_attention_cases()
    assert set(cases) == {"two_tokens", "three_tokens"}
    for name, (h, out) in cases.items():
        np.testing.assert_allclose(hash_fn.sparse_attention(np.array(h)), np.array(out), atol=1e-14, err_msg=name)


def test_attention_of_well_separated_rows_returns_each_row():
    """Mutually orthogonal rows of squared length >= 1: a token's score with itself leads every
    other score (all 0) by at least 1, so its SparseMax weights are one-hot and it gets its own row
    back.  SoftMax weights, or scores divided by sqrt(C), would mix rows in."""
    C = 6
    h = np.zeros((4, C))
    for t, (axis, length) in enumerate([(0, 1.0), (2, 1.2), (3, -1.5), (5, 3.0)]):
        h[t, axis] = length
    np.testing.assert_allclose(hash_fn.sparse_attention(h), h, atol=1e-15)
    # the control: with squared lengths below 1 the other rows do get weight
    assert np.abs(hash_fn.sparse_attention(0.5 * h) - 0.5 * h).max() > 0.05


def test_attention_of_a_zero_query_is_the_mean_of_the_rows():
    """A zero row scores 0 against every position: uniform weights 1/T, so its output is the plain
    mean of the value rows (which must be the rows of h themselves, all T of them)."""
    rng = np.random.default_rng(11)
    h = rng.standard_normal((5, 3))
    h[2] = 0.0
    np.testing.assert_allclose(hash_fn.sparse_attention(h)[2], h.mean(axis=0), atol=1e-15)


def test_attention_does_not_depend_on_the_order_of_the_other_tokens():
    """Token t's output is a function of the set of rows: permuting the sequence permutes the outputs."""
    rng = np.random.default_rng(12)
    h = rng.standard_normal((7, 4)) * 0.8
    perm = rng.permutation(7)
    np.testing.assert_allclose(hash_fn.sparse_attention(h[perm]), hash_fn.sparse_attention(h)[perm], atol=1e-13)


def test_forward_for_a_sequence_uses_the_attention_over_the_second_lstm_layer():
    """Whole forward on T > 1 with an output layer that reads the residual sum back out: with
    w_out = identity rows and b_out = 0 the logits ARE r = attention(h2) + c0, so
    log(probs) differences recover r up to a constant per token."""
    rng = np.random.default_rng(13)
    d, C, T = 5, 4, 6
    p = random_params(rng, d, C, 1, C, scale=0.6)
    p["w_out"] = np.eye(C)
    p["b_out"] = np.zeros(C)
    x = rng.standard_normal((T, d))
    _, _, probs = hash_fn.hash_forward(p, x, 1, C, 1)
    c0 = x @ p["w_in"].T + p["b_in"]
    ref = torch.nn.LSTM(C, C, num_layers=2, batch_first=True).double()
    with torch.no_grad():
        for n, key in (("weight_ih_l0", "w_ih1"), ("weight_hh_l0", "w_hh1"), ("bias_ih_l0", "b_ih1"), ("bias_hh_l0", "b_hh1"),
                       ("weight_ih_l1", "w_ih2"), ("weight_hh_l1", "w_hh2"), ("bias_ih_l1", "b_ih2"), ("bias_hh_l1", "b_hh2")):
            getattr(ref, n).copy_(torch.from_numpy(p[key]))
        h2 = ref(torch.from_numpy(c0)[None])[0][0].numpy()
    # attention by the exhaustive-search projection, not by the oracle's sparsemax
    att = np.stack([sum(w * h2[u] for u, w in enumerate(project_by_exhaustive_search(list(h2 @ h2[t])))) for t in range(T)])
    r = att + c0
    logp = np.log(probs[0])
    np.testing.assert_allclose(logp - logp[:, :1], r - r[:, :1], atol=1e-9)
