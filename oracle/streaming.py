"""fp64 oracle: attention of a "streaming" head (the head-wise sparsity extension, Appendix E).

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed.  Appendix E ("Efficient Management of KV cache") splits the heads of a layer into retrieval
heads, which keep every token and are evaluated exactly (oracle/attention.py), and streaming heads, which keep
only recent tokens and therefore never leave the GPU; Table 14 evaluates it with the streaming heads of
DuoAttention, whose heads keep a few initial "sink" tokens besides the recent ones.  The paper prints no formula
for it, so the reading taken here is the plain masked definition: a streaming head with parameters
(n_sink, n_recent) evaluates Eq. 3 over the visible keys only,

    visible(i) = { j <= i :  j < n_sink  or  i - j < n_recent },

i.e. the first n_sink tokens plus the n_recent most recent ones, the query's own token included.  n_sink = 0,
n_recent = 1 is the paper's literal sentence (only the most recent token is retained), and n_recent > i makes
the row identical to the exact one.

`attn_rows_streaming` is that definition written out.  `StreamingCache` is the data structure the definition
implies - a store that really holds only n_sink + n_recent rows per head, new rows overwriting the oldest recent
one - with `prefill_chunked_streaming` / `decode_step_streaming` evaluating Algorithm 1's order on it; that the
bounded store gives the same numbers as the mask over the full history is one of the pins.

Pins (tests/test_oracle_streaming.py): brute force with an explicit mask matrix and no max subtraction; a window
covering the whole history == the exact oracle; (0, 1) => the token's own value row; constant keys => mean of the
visible value rows; rows outside the visible set have no effect, rows inside do; torch's fp64
scaled_dot_product_attention with the same boolean mask; bounded store == mask over the full history; decode
step == last row.
"""
from __future__ import annotations

import math

import numpy as np


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def visible_mask(positions, n_keys: int, n_sink: int, n_recent: int) -> np.ndarray:
    """Boolean [R, n_keys]: key j is visible to the query at absolute position positions[r]."""
    assert n_sink >= 0 and n_recent >= 1
    i = np.asarray(positions, dtype=np.int64)[:, None]
    j = np.arange(n_keys, dtype=np.int64)[None, :]
    return (j <= i) & ((j < n_sink) | (i - j < n_recent))


def attn_rows_streaming(q_rows, K, V, positions, n_sink: int, n_recent: int) -> np.ndarray:
    """Outputs of selected query rows of ONE query head of a streaming head against the head's FULL history
    K, V [n, d] (row j = token j); only visible keys take part.  Returns float64 [R, d]."""
    q_rows, K, V = _f64(q_rows), _f64(K), _f64(V)
    positions = np.asarray(positions, dtype=np.int64)
    R, d_k = q_rows.shape
    assert K.shape == V.shape and K.shape[1] == d_k
    assert positions.shape == (R,) and (positions >= 0).all() and (positions < K.shape[0]).all()
    out = np.empty((R, V.shape[1]), dtype=np.float64)
    for r in range(R):
        vis = np.flatnonzero(visible_mask(positions[r:r + 1], K.shape[0], n_sink, n_recent)[0])
        s = (K[vis] @ q_rows[r]) / math.sqrt(d_k)
        w = np.exp(s - s.max())
        out[r] = (w / w.sum()) @ V[vis]
    return out


def attn_head_streaming(Q, K, V, past_len: int, n_sink: int, n_recent: int) -> np.ndarray:
    """All rows of one streaming KV head's query group: Q [G, C, d] at positions past_len..past_len+C-1 against
    the full history K, V [past_len + C, d].  Returns [G, C, d]."""
    Q = _f64(Q)
    G, C, _ = Q.shape
    pos = past_len + np.arange(C)
    return np.stack([attn_rows_streaming(Q[g], K, V, pos, n_sink, n_recent) for g in range(G)])


class StreamingCache:
    """The bounded store of one streaming head: n_sink sink rows, then n_recent recent rows kept as a ring in
    which token j >= n_sink lives in slot (j - n_sink) mod n_recent.  It never holds more than
    n_sink + n_recent rows, whatever the context length."""

    def __init__(self, head_dim: int, n_sink: int, n_recent: int):
        assert n_sink >= 0 and n_recent >= 1
        self.n_sink, self.n_recent = n_sink, n_recent
        self.K = np.zeros((n_sink + n_recent, head_dim))
        self.V = np.zeros((n_sink + n_recent, head_dim))
        self.pos = np.full(n_sink + n_recent, -1, dtype=np.int64)   # absolute position held by each slot
        self.length = 0                                              # tokens seen so far

    def slot_of(self, j: int) -> int:
        return j if j < self.n_sink else self.n_sink + (j - self.n_sink) % self.n_recent

    def append(self, k_row, v_row):
        s = self.slot_of(self.length)
        self.K[s], self.V[s], self.pos[s] = _f64(k_row), _f64(v_row), self.length
        self.length += 1

    def attend(self, q_row) -> np.ndarray:
        """Attention of the newest token's query over everything the store holds (append first)."""
        held = np.flatnonzero(self.pos >= 0)
        s = (self.K[held] @ _f64(q_row)) / math.sqrt(self.K.shape[1])
        w = np.exp(s - s.max())
        return (w / w.sum()) @ self.V[held]


def prefill_chunked_streaming(cache: StreamingCache, Q, K, V, chunk: int) -> np.ndarray:
    """Algorithm 1's prefill order for one streaming head on the bounded store: per chunk, every row sees the
    store as it was when the chunk began plus the chunk's own rows up to itself, restricted to its visible
    set; then the chunk's rows enter the store.  Q [G, S, d]; K, V [S, d].  Returns [G, S, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    G, S, d = Q.shape
    out = np.empty_like(Q)
    for c0 in range(0, S, chunk):
        c1 = min(S, c0 + chunk)
        held = np.flatnonzero(cache.pos >= 0)
        Kc = np.concatenate([cache.K[held], K[c0:c1]], axis=0)
        Vc = np.concatenate([cache.V[held], V[c0:c1]], axis=0)
        pc = np.concatenate([cache.pos[held], np.arange(c0, c1)])
        for i in range(c0, c1):
            vis = np.flatnonzero((pc <= i) & ((pc < cache.n_sink) | (i - pc < cache.n_recent)))
            for g in range(G):
                s = (Kc[vis] @ Q[g, i]) / math.sqrt(d)
                w = np.exp(s - s.max())
                out[g, i] = (w / w.sum()) @ Vc[vis]
        for j in range(c0, c1):
            cache.append(K[j], V[j])
    return out


def decode_step_streaming(cache: StreamingCache, q, k_new, v_new) -> np.ndarray:
    """Algorithm 1's decode step for one streaming head: the token's row enters the store (overwriting the row
    that just left the window), then its G query rows attend over the whole store.  q [G, d]."""
    cache.append(k_new, v_new)
    return np.stack([cache.attend(qg) for qg in _f64(q)])
