"""fp64 oracle: exact causal grouped-query attention, and the head-wise / chunked evaluation order.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed.  The method is claimed to be mathematically identical to standard attention
(Section 1, "exact mathematical equivalence"; Section 5, "unchanged behavior"), so the oracle is the plain
definition, written out:

    A_t = Softmax(Q_t K_cache^T / sqrt(d_k)) V_cache                      (Eq. 3)
    A_t^(h) evaluated independently per head h and concatenated           (Eq. 7-9)

with K_cache = [K_1..K_t] (Eq. 2), i.e. the query at absolute position p sees keys 0..p inclusive.
Grouped-query sharing: query heads [h*G, (h+1)*G) use KV head h; the offloaded unit is the KV head.

`HeadwiseCache` + `prefill_chunked` + `decode_step` follow Algorithm 1's order (chunk -> layer -> head
for prefill, token -> layer -> head for decode; per head: append the new K/V rows, then attend) with a cache
that grows chunk by chunk, which is the evaluation the paper says equals the monolithic one.

All inputs are widened to float64; all arithmetic is float64; numpy's matmul is the only library step.
Pins (tests/test_oracle_attention.py): brute-force evaluation without max-subtraction on tiny inputs,
rows of softmax weights summing to one, constant keys => running mean of V, causality, chunked/head-wise
== monolithic, single-key and dominant-key limits, permutation invariance of past (K,V) pairs, GQA sharing.
The paper prints no worked numeric attention output, so absolute values are pinned by those properties only.
"""
from __future__ import annotations

import math

import numpy as np


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def softmax_weights(q_row, K, n_keys: int) -> np.ndarray:
    """Softmax weights of one query row over keys 0..n_keys-1 (Eq. 3 with d_k = K.shape[1])."""
    q_row, K = _f64(q_row), _f64(K)
    d_k = K.shape[1]
    s = (K[:n_keys] @ q_row) / math.sqrt(d_k)
    e = np.exp(s - s.max())
    return e / e.sum()


def attn_rows(q_rows, K, V, positions) -> np.ndarray:
    """Attention outputs of selected query rows of ONE query head against ONE KV head.

    q_rows [R, d]; K, V [n, d] (row j = token j); positions [R] absolute token positions, row r sees keys
    0..positions[r] inclusive (Eq. 2-3).  Returns float64 [R, d].
    """
    q_rows, K, V = _f64(q_rows), _f64(K), _f64(V)
    positions = np.asarray(positions, dtype=np.int64)
    R, d_k = q_rows.shape
    assert K.shape == V.shape and K.shape[1] == d_k
    assert positions.shape == (R,) and (positions >= 0).all() and (positions < K.shape[0]).all()
    out = np.empty((R, V.shape[1]), dtype=np.float64)
    if R == 0:
        return out
    n_max = int(positions.max()) + 1
    scores = (q_rows @ K[:n_max].T) / math.sqrt(d_k)            # [R, n_max]
    cols = np.arange(n_max)[None, :]
    scores = np.where(cols <= positions[:, None], scores, -np.inf)
    scores -= scores.max(axis=1, keepdims=True)
    w = np.exp(scores)
    w /= w.sum(axis=1, keepdims=True)
    out[:] = w @ V[:n_max]
    return out


def attn_head(Q, K, V, past_len: int = 0) -> np.ndarray:
    """All rows of one KV head's query group.  Q [G, C, d] at positions past_len..past_len+C-1;
    K, V [past_len + C, d].  Returns [G, C, d]."""
    Q = _f64(Q)
    G, C, _ = Q.shape
    pos = past_len + np.arange(C)
    return np.stack([attn_rows(Q[g], K, V, pos) for g in range(G)])


def attn_layer(Q, K, V) -> np.ndarray:
    """Monolithic causal GQA attention of one layer.  Q [Hq, S, d]; K, V [Hkv, S, d]; returns [Hq, S, d]
    (the concatenation of the per-head outputs of Eq. 9, kept as a leading head axis)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    Hq, Hkv = Q.shape[0], K.shape[0]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    out = np.empty_like(Q)
    for h in range(Hkv):
        out[h * G:(h + 1) * G] = attn_head(Q[h * G:(h + 1) * G], K[h], V[h])
    return out


class HeadwiseCache:
    """The head-wise partitioned cache of Eq. 7-8: one growing (K, V) pair per (layer, KV head)."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int):
        self.K = [[np.zeros((0, head_dim)) for _ in range(n_kv_heads)] for _ in range(n_layers)]
        self.V = [[np.zeros((0, head_dim)) for _ in range(n_kv_heads)] for _ in range(n_layers)]

    def length(self, layer: int, head: int) -> int:
        return self.K[layer][head].shape[0]

    def update(self, layer: int, head: int, k_new, v_new):
        """Append rows (Eq. 2) and return the whole history of that head."""
        self.K[layer][head] = np.concatenate([self.K[layer][head], _f64(k_new)], axis=0)
        self.V[layer][head] = np.concatenate([self.V[layer][head], _f64(v_new)], axis=0)
        return self.K[layer][head], self.V[layer][head]


def prefill_chunked(cache: HeadwiseCache, Q, K, V, chunk: int) -> np.ndarray:
    """Algorithm 1, prefill phase.  Q [L, Hq, S, d]; K, V [L, Hkv, S, d]; chunks of `chunk` rows (the last
    may be short).  Loop order chunk -> layer -> head; per head: append, then attend.  Returns [L, Hq, S, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L, Hq, S, _ = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.empty_like(Q)
    for c0 in range(0, S, chunk):
        c1 = min(S, c0 + chunk)
        for layer in range(L):
            for h in range(Hkv):
                past = cache.length(layer, h)
                Kh, Vh = cache.update(layer, h, K[layer, h, c0:c1], V[layer, h, c0:c1])
                out[layer, h * G:(h + 1) * G, c0:c1] = attn_head(Q[layer, h * G:(h + 1) * G, c0:c1], Kh, Vh, past)
    return out


def decode_step(cache: HeadwiseCache, q, k_new, v_new) -> np.ndarray:
    """Algorithm 1, decode phase, one token.  q [L, Hq, d]; k_new, v_new [L, Hkv, d].  The new row is appended
    first, so the token attends to itself.  Returns [L, Hq, d]."""
    q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
    L, Hq, _ = q.shape
    Hkv = k_new.shape[1]
    G = Hq // Hkv
    out = np.empty_like(q)
    for layer in range(L):
        for h in range(Hkv):
            Kh, Vh = cache.update(layer, h, k_new[layer, h][None, :], v_new[layer, h][None, :])
            p = Kh.shape[0] - 1
            for g in range(G):
                out[layer, h * G + g] = attn_rows(q[layer, h * G + g][None, :], Kh, Vh, [p])[0]
    return out
