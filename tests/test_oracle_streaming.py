"""Pins of oracle/streaming.py (streaming heads of the head-wise sparsity extension, Appendix E) against things
fixed by the mathematics and by the already pinned exact oracle, not by the streaming oracle itself."""
import math

import numpy as np
import pytest

from oracle import attention as oa
from oracle import streaming as os_


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def brute_force_streaming(Q, K, V, n_sink, n_recent):
    """Independent formulation: S x S mask matrix written as three separate conditions, exp(s) / sum(exp(s))
    without max subtraction, exactly rounded sums, pure Python loops.  Q [G, S, d], K, V [S, d]."""
    G, S, d = Q.shape
    out = np.zeros((G, S, V.shape[1]))
    for g in range(G):
        for i in range(S):
            e = [0.0] * S
            for j in range(S):
                causal = j <= i
                is_sink = j < n_sink
                is_recent = j >= i - n_recent + 1
                if causal and (is_sink or is_recent):
                    e[j] = math.exp(math.fsum(Q[g, i, k] * K[j, k] for k in range(d)) / math.sqrt(d))
            z = math.fsum(e)
            for c in range(V.shape[1]):
                out[g, i, c] = math.fsum(e[j] * V[j, c] for j in range(S)) / z
    return out


@pytest.mark.parametrize("S,d,n_sink,n_recent", [(19, 4, 0, 1), (19, 4, 3, 5), (33, 8, 4, 7), (12, 4, 20, 3), (25, 4, 0, 6)])
def test_s1_brute_force(S, d, n_sink, n_recent):
    rng = np.random.default_rng(300 + S + n_sink)
    Q, K, V = _rand(rng, 2, S, d), _rand(rng, S, d), _rand(rng, S, d)
    ref = brute_force_streaming(Q, K, V, n_sink, n_recent)
    got = os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent)
    assert np.max(np.abs(got - ref)) <= 1e-13


def test_s2_window_covering_the_history_is_the_exact_oracle():
    rng = np.random.default_rng(302)
    S, d = 70, 8
    Q, K, V = _rand(rng, 3, S, d), _rand(rng, S, d), _rand(rng, S, d)
    exact = oa.attn_head(Q, K, V)
    for n_sink, n_recent in [(0, S), (0, S + 100), (5, S), (S, 1), (S + 3, 2)]:
        got = os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent)
        assert np.max(np.abs(got - exact)) <= 1e-14
    # a short window agrees with the exact oracle on exactly the rows whose whole history is still visible
    n_sink, n_recent = 4, 9
    got = os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent)
    whole = np.arange(S) < n_sink + n_recent
    assert np.max(np.abs(got[:, whole] - exact[:, whole])) <= 1e-14
    assert np.min(np.max(np.abs(got[:, ~whole] - exact[:, ~whole]), axis=(0, 2))) > 1e-9


def test_s3_most_recent_token_only_returns_its_value_row():
    """The paper's literal sentence: a streaming head that retains only the most recent token."""
    rng = np.random.default_rng(303)
    S, d = 21, 8
    Q, K, V = _rand(rng, 2, S, d), _rand(rng, S, d), _rand(rng, S, d)
    got = os_.attn_head_streaming(Q, K, V, 0, 0, 1)
    assert np.max(np.abs(got - V[None])) <= 1e-15


def test_s4_constant_keys_give_the_mean_of_the_visible_values():
    rng = np.random.default_rng(304)
    S, d, n_sink, n_recent = 60, 8, 3, 10
    K = np.tile(_rand(rng, 1, d), (S, 1))
    V = _rand(rng, S, d)
    Q = _rand(rng, 2, S, d)
    got = os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent)
    for i in range(S):
        vis = sorted(set(range(min(n_sink, i + 1))) | set(range(max(0, i - n_recent + 1), i + 1)))
        assert np.max(np.abs(got[:, i] - V[vis].mean(axis=0)[None])) <= 1e-13


def test_s5_rows_outside_the_visible_set_have_no_effect_rows_inside_do():
    rng = np.random.default_rng(305)
    S, d, n_sink, n_recent, i = 80, 8, 4, 12, 57
    Q, K, V = _rand(rng, 2, S, d), _rand(rng, S, d), _rand(rng, S, d)
    base = os_.attn_rows_streaming(Q[0, i][None], K, V, [i], n_sink, n_recent)
    hidden = [j for j in range(S) if not (j <= i and (j < n_sink or i - j < n_recent))]
    assert n_sink in hidden and (i - n_recent) in hidden and (i + 1) in hidden
    K2, V2 = K.copy(), V.copy()
    K2[hidden] += 100.0
    V2[hidden] -= 100.0
    assert np.array_equal(os_.attn_rows_streaming(Q[0, i][None], K2, V2, [i], n_sink, n_recent), base)
    for j in (0, n_sink - 1, i - n_recent + 1, i):        # the four edges of the visible set
        V3 = V.copy()
        V3[j] += 1.0
        assert np.max(np.abs(os_.attn_rows_streaming(Q[0, i][None], K, V3, [i], n_sink, n_recent) - base)) > 1e-6


def test_s6_library_routine_with_the_same_boolean_mask():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(306)
    G, S, d, n_sink, n_recent, P = 4, 90, 16, 5, 17, 31
    Q, K, V = _rand(rng, G, S, d), _rand(rng, S, d), _rand(rng, S, d)
    i = torch.arange(S)[:, None]
    j = torch.arange(S)[None, :]
    mask = (j <= i) & ((j < n_sink) | (j > i - n_recent))
    tq, tk, tv = torch.from_numpy(Q), torch.from_numpy(K).expand(G, S, d), torch.from_numpy(V).expand(G, S, d)
    ref = F.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=mask)[0].numpy()
    np.testing.assert_allclose(os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent), ref, rtol=0, atol=1e-12)
    # a chunk behind a past
    got = os_.attn_head_streaming(Q[:, P:], K, V, P, n_sink, n_recent)
    np.testing.assert_allclose(got, ref[:, P:], rtol=0, atol=1e-12)


@pytest.mark.parametrize("n_sink,n_recent,chunk", [(0, 1, 5), (3, 5, 4), (3, 5, 11), (6, 16, 7), (40, 4, 9), (2, 64, 13)])
def test_s7_bounded_store_equals_the_mask_over_the_full_history(n_sink, n_recent, chunk):
    """The store never holds more than n_sink + n_recent rows, yet chunked prefill and decode on it give the
    numbers of the masked definition evaluated with the whole history at hand."""
    rng = np.random.default_rng(307 + n_sink)
    G, S, T, d = 2, 37, 9, 8
    Q, K, V = _rand(rng, G, S + T, d), _rand(rng, S + T, d), _rand(rng, S + T, d)
    ref = os_.attn_head_streaming(Q, K, V, 0, n_sink, n_recent)
    cache = os_.StreamingCache(d, n_sink, n_recent)
    got = os_.prefill_chunked_streaming(cache, Q[:, :S], K[:S], V[:S], chunk)
    assert cache.K.shape[0] == n_sink + n_recent
    np.testing.assert_allclose(got, ref[:, :S], rtol=0, atol=1e-13)
    for t in range(S, S + T):
        out = os_.decode_step_streaming(cache, Q[:, t], K[t], V[t])
        np.testing.assert_allclose(out, ref[:, t], rtol=0, atol=1e-13)
    # what the store holds at the end is exactly the visible set of the next token minus that token
    held = sorted(cache.pos[cache.pos >= 0].tolist())
    n = S + T
    want = sorted(set(range(min(n_sink, n))) | set(range(max(n_sink, n - n_recent), n)))
    assert held == want


def test_s8_visible_mask_counts():
    for n_sink, n_recent in [(0, 1), (4, 8), (16, 3)]:
        m = os_.visible_mask(np.arange(50), 50, n_sink, n_recent)
        for i in range(50):
            want = min(i + 1, n_recent) + max(0, min(n_sink, i - n_recent + 1))
            assert m[i].sum() == want
            assert m[i, i] and not m[i, i + 1:].any()
