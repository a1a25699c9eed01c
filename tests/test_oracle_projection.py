"""Pins of oracle/projection.py (Eq. 1 projections, rotary position embedding, output projection) against things
fixed by the mathematics, not by the oracle itself."""
import cmath
import math

import numpy as np
import pytest

from oracle import projection as op


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_p1_exactly_rounded_loops():
    """Independent formulation: pure Python loops, math.fsum, the rotation written as a 2 x 2 matrix per pair."""
    rng = np.random.default_rng(401)
    n, D, d, Hq, Hkv, theta, P = 5, 6, 4, 2, 1, 10000.0, 7
    X, Wq, Wk, Wv = _rand(rng, n, D), _rand(rng, Hq * d, D), _rand(rng, Hkv * d, D), _rand(rng, Hkv * d, D)
    Q, K, V = op.qkv_rope(X, Wq, Wk, Wv, np.arange(P, P + n), d, theta)

    def ref(W, H, rotate):
        out = np.zeros((H, n, d))
        for h in range(H):
            for t in range(n):
                y = [math.fsum(X[t, k] * W[h * d + j, k] for k in range(D)) for j in range(d)]
                if rotate:
                    for i in range(d // 2):
                        a = (P + t) * theta ** (-2.0 * i / d)
                        lo, hi = y[i], y[i + d // 2]
                        y[i] = math.cos(a) * lo - math.sin(a) * hi
                        y[i + d // 2] = math.sin(a) * lo + math.cos(a) * hi
                out[h, t] = y
        return out

    assert np.max(np.abs(Q - ref(Wq, Hq, True))) <= 1e-13
    assert np.max(np.abs(K - ref(Wk, Hkv, True))) <= 1e-13
    assert np.max(np.abs(V - ref(Wv, Hkv, False))) <= 1e-13


def test_p2_identity_weights_return_the_hidden_states_slices():
    rng = np.random.default_rng(402)
    n, d, Hq, Hkv = 6, 8, 4, 2
    D = Hq * d
    X = _rand(rng, n, D)
    Wq = np.eye(D)
    Wk = np.eye(D)[:Hkv * d]
    Wv = np.eye(D)[Hkv * d:2 * Hkv * d]
    Q, K, V = op.qkv_rope(X, Wq, Wk, Wv, np.arange(n), d, None)
    for h in range(Hq):
        assert np.array_equal(Q[h], X[:, h * d:(h + 1) * d])
    for h in range(Hkv):
        assert np.array_equal(K[h], X[:, h * d:(h + 1) * d])
        assert np.array_equal(V[h], X[:, (Hkv + h) * d:(Hkv + h + 1) * d])


def test_p3_rotation_is_multiplication_of_the_complex_pair():
    rng = np.random.default_rng(403)
    d, theta = 16, 500000.0
    pos = np.array([0, 1, 2, 77, 1048575])
    x = _rand(rng, len(pos), d)
    got = op.apply_rope(x, pos, theta)
    for t, p in enumerate(pos):
        for i in range(d // 2):
            z = complex(x[t, i], x[t, i + d // 2]) * cmath.exp(1j * float(p) * theta ** (-2.0 * i / d))
            assert abs(got[t, i] - z.real) <= 1e-9 and abs(got[t, i + d // 2] - z.imag) <= 1e-9
    # first pair has frequency 1: the unit vector at position p lands at (cos p, sin p)
    e = np.zeros((1, d)); e[0, 0] = 1.0
    r = op.apply_rope(e, [3], theta)
    assert abs(r[0, 0] - math.cos(3.0)) <= 1e-15 and abs(r[0, d // 2] - math.sin(3.0)) <= 1e-15


def test_p4_position_zero_identity_norms_and_composition():
    rng = np.random.default_rng(404)
    d, theta, n = 32, 10000.0, 9
    x = _rand(rng, 3, n, d)
    assert np.array_equal(op.apply_rope(x, np.zeros(n), theta), x)
    pos = np.arange(100, 100 + n)
    y = op.apply_rope(x, pos, theta)
    pair = lambda a: a[..., :d // 2] ** 2 + a[..., d // 2:] ** 2
    assert np.max(np.abs(pair(y) - pair(x))) <= 1e-12
    z = op.apply_rope(op.apply_rope(x, pos, theta), 2 * pos + 5, theta)
    assert np.max(np.abs(z - op.apply_rope(x, 3 * pos + 5, theta))) <= 1e-10


def test_p5_scores_depend_on_the_position_difference_only():
    rng = np.random.default_rng(405)
    d, theta = 64, 500000.0
    q, k = _rand(rng, 1, d), _rand(rng, 1, d)
    for m, n in [(10, 3), (1000, 993), (123456, 123449)]:
        s = op.apply_rope(q, [m], theta)[0] @ op.apply_rope(k, [n], theta)[0]
        s0 = op.apply_rope(q, [m - n], theta)[0] @ k[0]
        assert abs(s - s0) <= 1e-8


def test_p6_library_routine_linear():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(406)
    n, D, d, Hq, Hkv = 11, 24, 8, 3, 1
    X, Wq, Wk, Wv = _rand(rng, n, D), _rand(rng, Hq * d, D), _rand(rng, Hkv * d, D), _rand(rng, Hkv * d, D)
    Q, K, V = op.qkv_rope(X, Wq, Wk, Wv, np.arange(n), d, None)
    lin = lambda W: torch.nn.functional.linear(torch.from_numpy(X), torch.from_numpy(W)).numpy()
    np.testing.assert_allclose(Q.transpose(1, 0, 2).reshape(n, -1), lin(Wq), rtol=0, atol=1e-12)
    np.testing.assert_allclose(K.transpose(1, 0, 2).reshape(n, -1), lin(Wk), rtol=0, atol=1e-12)
    np.testing.assert_allclose(V.transpose(1, 0, 2).reshape(n, -1), lin(Wv), rtol=0, atol=1e-12)
    A, Wo = _rand(rng, Hq, n, d), _rand(rng, D, Hq * d)
    ref = torch.nn.functional.linear(torch.from_numpy(A.transpose(1, 0, 2).reshape(n, -1).copy()),
                                     torch.from_numpy(Wo)).numpy()
    np.testing.assert_allclose(op.out_proj(A, Wo), ref, rtol=0, atol=1e-12)


def test_p7_output_projection_of_identity_is_the_concatenation_of_heads():
    rng = np.random.default_rng(407)
    Hq, n, d = 3, 5, 4
    A = _rand(rng, Hq, n, d)
    Y = op.out_proj(A, np.eye(Hq * d))
    for h in range(Hq):
        assert np.array_equal(Y[:, h * d:(h + 1) * d], A[h])
    # brute force with a dense weight
    Wo = _rand(rng, 7, Hq * d)
    Y = op.out_proj(A, Wo)
    for t in range(n):
        for o in range(7):
            ref = math.fsum(A[h, t, j] * Wo[o, h * d + j] for h in range(Hq) for j in range(d))
            assert abs(Y[t, o] - ref) <= 1e-13
