"""fp64 oracle: the steps either side of head-wise attention - Q/K/V projection (with rotary position embedding)
into head-major layout, and the output projection of the concatenated heads.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed.  Section 3.1, Eq. 1: the key and the value of a token are linear projections of its hidden
state, K_t = W_K E(x_t), V_t = W_V E(x_t) (the query likewise); Appendix F's attention module calls them q_proj,
k_proj, v_proj, views the results as [tokens][heads][head_dim] and hands each head's slice to the head-wise cache;
Eq. 9 concatenates the head outputs, which the model's output projection then consumes.  The evaluated model
(Llama-3-8B, Section 6) rotates queries and keys by their position before attention (rotary position embedding,
cited in Section 7); the paper prints no formula for it, so the reading taken is the standard one in that model's
convention: within a head of dimension d, dimension i < d/2 is paired with i + d/2, and the pair of the token at
position p is rotated by the angle p * theta^(-2i/d).

All inputs are widened to float64; numpy's matmul is the only library step.  Weights use the [out_features,
in_features] layout (y = x W^T).
Pins (tests/test_oracle_projection.py): exactly rounded loop evaluation on tiny shapes; identity weights return
the hidden state's own slices; rotation as multiplication by exp(i p theta_i) of the complex pair; position 0 is
the identity; pair norms are preserved; rotations compose additively; q.k after rotation depends on the position
difference only; torch's fp64 linear; the output projection of one-hot weights is Eq. 9's concatenation.
"""
from __future__ import annotations

import numpy as np


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def rope_angles(positions, head_dim: int, theta: float) -> np.ndarray:
    """[n, head_dim / 2] rotation angles p * theta^(-2i / head_dim)."""
    half = head_dim // 2
    inv_freq = np.float64(theta) ** (-np.arange(half, dtype=np.float64) * 2.0 / head_dim)
    return np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]


def apply_rope(x, positions, theta: float) -> np.ndarray:
    """x [..., n, d] with rows at the given absolute positions; pairs (i, i + d/2) rotated by the row's angles."""
    x = _f64(x)
    d = x.shape[-1]
    half = d // 2
    ang = rope_angles(positions, d, theta)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def qkv_rope(X, Wq, Wk, Wv, positions, head_dim: int, theta: float | None):
    """Eq. 1 for a block of tokens, head-major.  X [n, D]; Wq [Hq*d, D], Wk and Wv [Hkv*d, D]; positions [n].
    Returns Q [Hq, n, d], K [Hkv, n, d] (both rotated unless theta is None) and V [Hkv, n, d]."""
    X, Wq, Wk, Wv = _f64(X), _f64(Wq), _f64(Wk), _f64(Wv)
    n = X.shape[0]

    def heads(W):
        y = X @ W.T                                            # [n, H*d]
        return y.reshape(n, W.shape[0] // head_dim, head_dim).transpose(1, 0, 2)

    Q, K, V = heads(Wq), heads(Wk), heads(Wv)
    if theta is not None:
        Q, K = apply_rope(Q, positions, theta), apply_rope(K, positions, theta)
    return Q, K, V


def out_proj(A, Wo) -> np.ndarray:
    """Output projection of the concatenated heads (Eq. 9's Concat, then a linear map).  A [Hq, n, d] head-major
    attention outputs; Wo [D, Hq*d].  Returns [n, D]."""
    A, Wo = _f64(A), _f64(Wo)
    Hq, n, d = A.shape
    concat = A.transpose(1, 0, 2).reshape(n, Hq * d)
    return concat @ Wo.T
