"""CPU oracle of the hash function that predicts expert ids and scaling factors (Section 3.4.2).
TEST INFRASTRUCTURE ONLY, like the rest of this package.

The paper describes the network in words: a fully connected layer that compresses the embedding
dimension, a 2-layer LSTM, an attention layer over the LSTM's output sequence (query = key =
value = that sequence, dot-product score) whose weights go through SparseMax instead of SoftMax, a
residual connection "right before the final fully connected layer", and that final layer; the
output is, per MoE layer and token, the experts to activate and their scaling factor alpha
(Section 3.1, Algorithm 1 right column: one prediction h_l per layer l).  Everything the paper
leaves open is a reading, stated here and in the design notes:

* sizes: compressed width C = LSTM hidden width (so that the residual can add the two);
* LSTM cell: the standard one (input, forget, cell, output gates in this order; sigmoid, tanh),
  zero initial state, both bias vectors;
* attention: score(q, k) = q . k without scaling; SparseMax over the positions of the sequence;
* residual: attention output + the token's own compressed embedding ("the current token is always
  the most crucial");
* output layer: one linear head of E logits per MoE layer; scaling factor = SoftMax probability of
  the expert (the router's alpha is a SoftMax output, Section 3.1); the k largest are kept, ties
  to the lower expert id.

All arithmetic in float64, steps in the order above, no fusion.
Pins: tests/test_oracle_hash.py (SparseMax against an exhaustive search over supports and against
its defining properties; the LSTM against torch.nn.LSTM; the attention against hand-worked
sequences - one-hot weights for well separated rows, the plain mean for a zero query, a
two-token case from tests/golden/sparse_attention_2tok.txt; special cases of the whole forward)."""
from __future__ import annotations

import numpy as np


def sparsemax(z) -> np.ndarray:
    """Euclidean projection of z onto the probability simplex (the closed form of Martins and
    Astudillo): sort descending, k = max{j : 1 + j z_(j) > sum_{i<=j} z_(i)}, tau = (sum_{i<=k} z_(i) - 1) / k,
    p = max(z - tau, 0)."""
    z = np.asarray(z, dtype=np.float64)
    zs = np.sort(z)[::-1]
    cs = np.cumsum(zs)
    k = 0
    for j in range(1, len(z) + 1):
        if 1.0 + j * zs[j - 1] > cs[j - 1]:
            k = j
    tau = (cs[k - 1] - 1.0) / k
    return np.maximum(z - tau, 0.0)


def sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def lstm_layer(x, w_ih, w_hh, b_ih, b_hh) -> np.ndarray:
    """x [T, I] -> h [T, H]; gates stacked as (input, forget, cell, output) in the 4H rows."""
    x = np.asarray(x, dtype=np.float64)
    H = w_hh.shape[1]
    h = np.zeros(H)
    c = np.zeros(H)
    out = np.empty((x.shape[0], H))
    for t in range(x.shape[0]):
        g = w_ih @ x[t] + b_ih + w_hh @ h + b_hh
        i, f, gg, o = sigmoid(g[:H]), sigmoid(g[H:2 * H]), np.tanh(g[2 * H:3 * H]), sigmoid(g[3 * H:])
        c = f * c + i * gg
        h = o * np.tanh(c)
        out[t] = h
    return out


def sparse_attention(h) -> np.ndarray:
    """Attention of a sequence over itself with SparseMax weights (Section 3.4.2): query = key =
    value = h [T, C]; for token t the scores are the plain dot products h[u] . h[t] over the
    positions u of the sequence, the weights their SparseMax, the output the weighted sum of the
    rows h[u].  Returns [T, C]."""
    h = np.asarray(h, dtype=np.float64)
    out = np.empty_like(h)
    for t in range(h.shape[0]):
        scores = np.array([np.dot(h[u], h[t]) for u in range(h.shape[0])])
        w = sparsemax(scores)
        out[t] = sum(w[u] * h[u] for u in range(h.shape[0]))
    return out


def param_shapes(d_model: int, C: int, L: int, E: int):
    """Names and shapes of the parameters, in the order they are packed for the library."""
    return [("w_in", (C, d_model)), ("b_in", (C,)),
            ("w_ih1", (4 * C, C)), ("w_hh1", (4 * C, C)), ("b_ih1", (4 * C,)), ("b_hh1", (4 * C,)),
            ("w_ih2", (4 * C, C)), ("w_hh2", (4 * C, C)), ("b_ih2", (4 * C,)), ("b_hh2", (4 * C,)),
            ("w_out", (L * E, C)), ("b_out", (L * E,))]


def hash_forward(params: dict, x, L: int, E: int, k: int):
    """x: float [T, d_model] (one sequence).  Returns (ids int32 [L, T, k], alpha float64 [L, T, k],
    probs float64 [L, T, E]); probs is returned so that tests can judge near-ties."""
    p = {n: np.asarray(v, dtype=np.float64) for n, v in params.items()}
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    c0 = x @ p["w_in"].T + p["b_in"]                                     # compress the embedding
    h1 = lstm_layer(c0, p["w_ih1"], p["w_hh1"], p["b_ih1"], p["b_hh1"])
    h2 = lstm_layer(h1, p["w_ih2"], p["w_hh2"], p["b_ih2"], p["b_hh2"])
    att = sparse_attention(h2)                                           # over the sequence
    r = att + c0                                                         # residual before the last layer
    logits = r @ p["w_out"].T + p["b_out"]
    ids = np.empty((L, T, k), dtype=np.int32)
    alpha = np.empty((L, T, k))
    probs = np.empty((L, T, E))
    for l in range(L):
        z = logits[:, l * E:(l + 1) * E]
        e = np.exp(z - z.max(axis=1, keepdims=True))
        pr = e / e.sum(axis=1, keepdims=True)
        probs[l] = pr
        for t in range(T):
            order = sorted(range(E), key=lambda j: (-pr[t, j], j))[:k]
            ids[l, t] = order
            alpha[l, t] = pr[t, order]
    return ids, alpha, probs
