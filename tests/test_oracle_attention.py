"""Pins of oracle/attention.py against things fixed by the mathematics, not by the oracle itself."""
import math

import numpy as np
import pytest

from oracle import attention as oa


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def brute_force_layer(Q, K, V):
    """Independent formulation: full S x S score matrix per head, explicit -inf mask, exp(s)/sum(exp(s))
    without max subtraction, exactly rounded sums (math.fsum), pure Python loops."""
    Hq, S, d = Q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    out = np.zeros((Hq, S, V.shape[2]))
    for a in range(Hq):
        h = a // G
        for i in range(S):
            e = []
            for j in range(S):
                if j > i:
                    e.append(0.0)            # exp(-inf)
                else:
                    s = math.fsum(Q[a, i, k] * K[h, j, k] for k in range(d)) / math.sqrt(d)
                    e.append(math.exp(s))
            z = math.fsum(e)
            for c in range(V.shape[2]):
                out[a, i, c] = math.fsum(e[j] * V[h, j, c] for j in range(S)) / z
    return out


@pytest.mark.parametrize("G,S,d", [(1, 9, 4), (2, 17, 8), (4, 32, 8)])
def test_o1_brute_force(G, S, d):
    rng = np.random.default_rng(100 + G)
    Hkv = 2
    Q, K, V = _rand(rng, Hkv * G, S, d), _rand(rng, Hkv, S, d), _rand(rng, Hkv, S, d)
    ref = brute_force_layer(Q, K, V)
    got = oa.attn_layer(Q, K, V)
    assert np.max(np.abs(got - ref)) <= 1e-13


def test_o2_weights_sum_to_one_and_unit_values():
    rng = np.random.default_rng(2)
    S, d = 300, 16
    q, K = _rand(rng, d), _rand(rng, S, d)
    for n in (1, 2, 150, 300):
        w = oa.softmax_weights(q, K, n)
        assert w.shape == (n,) and abs(w.sum() - 1.0) <= 1e-14 and (w > 0).all()
    Q = _rand(rng, 2, S, d)
    out = oa.attn_head(Q, K, np.ones((S, d)))
    assert np.max(np.abs(out - 1.0)) <= 1e-14


def test_o3_constant_keys_give_running_mean_of_values():
    rng = np.random.default_rng(3)
    S, d = 65, 8
    K = np.tile(_rand(rng, 1, d), (S, 1))
    V = _rand(rng, S, d)
    Q = _rand(rng, 3, S, d)
    out = oa.attn_head(Q, K, V)
    running_mean = np.cumsum(V, axis=0) / np.arange(1, S + 1)[:, None]
    assert np.max(np.abs(out - running_mean[None])) <= 1e-13
    # a query orthogonal to every key gives the same uniform weights
    K2 = _rand(rng, S, d)
    K2[:, 0] = 0.0
    q = np.zeros((1, S, d)); q[..., 0] = 3.0
    assert np.max(np.abs(oa.attn_head(q, K2, V) - running_mean[None])) <= 1e-13


def test_o4_causality_future_rows_have_no_effect():
    rng = np.random.default_rng(4)
    S, d, i = 40, 8, 17
    Q, K, V = _rand(rng, 2, S, d), _rand(rng, S, d), _rand(rng, S, d)
    base = oa.attn_head(Q, K, V)
    K2, V2 = K.copy(), V.copy()
    K2[i + 1:] += 5.0 * _rand(rng, S - i - 1, d)
    V2[i + 1:] -= 7.0
    pert = oa.attn_head(Q, K2, V2)
    assert np.array_equal(pert[:, :i + 1], base[:, :i + 1])
    assert not np.allclose(pert[:, i + 1:], base[:, i + 1:])
    # the key at the query's own position does count (inclusive mask)
    K3 = K.copy(); K3[i] += 1.0
    assert not np.allclose(oa.attn_head(Q, K3, V)[:, i], base[:, i])


@pytest.mark.parametrize("chunk", [1, 5, 16, 64])
def test_o5_chunked_headwise_equals_monolithic(chunk):
    rng = np.random.default_rng(5)
    L, Hkv, G, S, d = 2, 2, 2, 37, 8
    Q, K, V = _rand(rng, L, Hkv * G, S, d), _rand(rng, L, Hkv, S, d), _rand(rng, L, Hkv, S, d)
    cache = oa.HeadwiseCache(L, Hkv, d)
    got = oa.prefill_chunked(cache, Q, K, V, chunk)
    ref = np.stack([oa.attn_layer(Q[l], K[l], V[l]) for l in range(L)])
    assert np.max(np.abs(got - ref)) <= 1e-12
    assert cache.length(1, 1) == S and np.array_equal(cache.K[1][1], K[1, 1])
    # decode: the new row is appended first and equals the next prefill row
    q1, k1, v1 = _rand(rng, L, Hkv * G, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    dec = oa.decode_step(cache, q1, k1, v1)
    Qx = np.concatenate([Q, q1[:, :, None]], axis=2)
    Kx = np.concatenate([K, k1[:, :, None]], axis=2)
    Vx = np.concatenate([V, v1[:, :, None]], axis=2)
    ref1 = np.stack([oa.attn_layer(Qx[l], Kx[l], Vx[l]) for l in range(L)])[:, :, -1]
    assert np.max(np.abs(dec - ref1)) <= 1e-12
    assert cache.length(0, 0) == S + 1


def test_o6_special_cases():
    rng = np.random.default_rng(6)
    d = 8
    # one key: the output is its value row
    q, k, v = _rand(rng, 1, d), _rand(rng, 1, d), _rand(rng, 1, d)
    assert np.array_equal(oa.attn_rows(q, k, v, [0]), v)
    # a key whose logit is 50 above the rest takes all the weight (to ~e^-50)
    S = 20
    K, V = 0.01 * _rand(rng, S, d), _rand(rng, S, d)
    qrow = np.zeros((1, d)); qrow[0, 0] = 1.0
    K[7, 0] = 50.0 * math.sqrt(d)
    assert np.max(np.abs(oa.attn_rows(qrow, K, V, [S - 1]) - V[7])) <= 1e-15 + 1e-18 * S
    # permuting the (K,V) pairs of the past leaves a decode row unchanged
    K, V, qrow = _rand(rng, S, d), _rand(rng, S, d), _rand(rng, 1, d)
    perm = rng.permutation(S)
    a = oa.attn_rows(qrow, K, V, [S - 1]); b = oa.attn_rows(qrow, K[perm], V[perm], [S - 1])
    assert np.max(np.abs(a - b)) <= 1e-14
    # identical queries in a group give identical outputs, distinct groups use distinct KV heads
    Hkv, G = 2, 4
    Q = np.tile(_rand(rng, Hkv, 1, S, d), (1, G, 1, 1)).reshape(Hkv * G, S, d)
    Kh, Vh = _rand(rng, Hkv, S, d), _rand(rng, Hkv, S, d)
    out = oa.attn_layer(Q, Kh, Vh)
    for h in range(Hkv):
        for g in range(1, G):
            assert np.array_equal(out[h * G + g], out[h * G])
    assert not np.allclose(out[0], out[G])
    # scale is 1/sqrt(d_k): doubling d by zero padding must change the weights accordingly
    w8 = oa.softmax_weights(qrow[0], K, S)
    Kpad = np.concatenate([K, np.zeros((S, 3 * d))], axis=1)
    qpad = np.concatenate([qrow[0], np.zeros(3 * d)])
    w32 = oa.softmax_weights(qpad, Kpad, S)
    s = (K @ qrow[0])
    ref8 = np.exp(s / math.sqrt(d)); ref8 /= ref8.sum()
    ref32 = np.exp(s / math.sqrt(4 * d)); ref32 /= ref32.sum()
    assert np.max(np.abs(w8 - ref8)) <= 1e-15 and np.max(np.abs(w32 - ref32)) <= 1e-15


def test_rows_match_full_and_positions_are_absolute():
    rng = np.random.default_rng(7)
    S, d, G = 50, 16, 2
    Q, K, V = _rand(rng, G, S, d), _rand(rng, S, d), _rand(rng, S, d)
    full = oa.attn_head(Q, K, V)
    pos = np.array([0, 1, 13, 49, 30])
    rows = oa.attn_rows(Q[1][pos], K, V, pos)
    assert np.max(np.abs(rows - full[1, pos])) <= 1e-15
    # chunk with a past: rows are at positions past..past+C-1
    past, C = 20, 30
    part = oa.attn_head(Q[:, past:], K, V, past_len=past)
    assert np.max(np.abs(part - full[:, past:])) <= 1e-15


def test_o7_library_routine_scaled_dot_product_attention():
    """Special case that is a library routine: torch's CPU scaled_dot_product_attention in fp64 (causal flag with no
    past; an explicit boolean mask for a chunk behind a past), with the KV heads repeated for the query groups."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(77)
    Hkv, G, S, d = 2, 4, 45, 16
    Q, K, V = _rand(rng, Hkv * G, S, d), _rand(rng, Hkv, S, d), _rand(rng, Hkv, S, d)
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, np.repeat(K, G, axis=0), np.repeat(V, G, axis=0)))
    ref = F.scaled_dot_product_attention(tq[None], tk[None], tv[None], is_causal=True)[0].numpy()
    np.testing.assert_allclose(oa.attn_layer(Q, K, V), ref, rtol=0, atol=1e-12)
    # rows [P, S) of head 1's group against keys [0, S): mask[i, j] = j <= P + i
    P = 29
    mask = torch.arange(S)[None, :] <= (P + torch.arange(S - P))[:, None]
    refp = F.scaled_dot_product_attention(tq[G:2 * G, P:][None], tk[G:2 * G][None], tv[G:2 * G][None],
                                          attn_mask=mask)[0].numpy()
    got = oa.attn_head(Q[G:2 * G, P:], K[1], V[1], past_len=P)
    np.testing.assert_allclose(got, refp, rtol=0, atol=1e-12)


def test_o8_decode_step_is_the_last_row_of_the_full_evaluation():
    rng = np.random.default_rng(78)
    L, Hkv, G, S, d = 1, 2, 2, 23, 8
    Q, K, V = _rand(rng, L, Hkv * G, S + 1, d), _rand(rng, L, Hkv, S + 1, d), _rand(rng, L, Hkv, S + 1, d)
    full = oa.attn_layer(Q[0], K[0], V[0])
    cache = oa.HeadwiseCache(L, Hkv, d)
    oa.prefill_chunked(cache, Q[:, :, :S], K[:, :, :S], V[:, :, :S], chunk=7)
    out = oa.decode_step(cache, Q[:, :, S], K[:, :, S], V[:, :, S])
    np.testing.assert_allclose(np.asarray(out)[0], full[:, S], rtol=0, atol=1e-12)
