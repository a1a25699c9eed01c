"""Pins of oracle/kvquant.py (4-bit rows on the host link; Appendix B's 4-bit KV representation composed with
head-wise offload) against things fixed by arithmetic and by the exact attention oracle, not by the code itself."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import attention as oa
from oracle import kvquant as kq


def _bf16(x):
    return kq.bf16_rne(np.asarray(x, dtype=np.float32))


def _rows(seed, n, d=128, spread=1.0):
    rng = np.random.default_rng(seed)
    return _bf16(rng.standard_normal((n, d)) * spread)


def test_k1_bf16_rounding_known_values():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to the even mantissa (1); 1 + 3 * 2^-8 is a tie that goes up
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 3.140625],
                 dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 3.140625], dtype=np.float32)
    assert np.array_equal(kq.bf16_rne(x), want)


def test_k2_error_bound_in_rational_arithmetic():
    """|x - x^| <= scale / 2 (rounding to a level) + 15 * |scale - range/15| (clipping when the stored scale was
    rounded down) + 2^-8 |x^| (x^ is rounded to bf16), evaluated exactly."""
    for seed, spread in [(1, 1.0), (2, 30.0), (3, 1e-3)]:
        x = _rows(seed, 7, spread=spread)
        codes, scale, zero = kq.quantize_rows(x)
        y = kq.dequantize_rows(codes, scale, zero)
        for r in range(x.shape[0]):
            for e in range(x.shape[1]):
                g = e // 32
                grp = x[r, g * 32:(g + 1) * 32]
                rng15 = (Fraction(float(grp.max())) - Fraction(float(grp.min()))) / 15
                s = Fraction(float(scale[r, g]))
                err = abs(Fraction(float(x[r, e])) - Fraction(float(y[r, e])))
                bound = s / 2 + 15 * abs(s - rng15) + abs(Fraction(float(y[r, e]))) / 256 + s / 2 ** 20
                assert err <= bound, (seed, r, e)
        assert codes.min() >= 0 and codes.max() <= 15


def test_k3_code_is_the_nearest_of_the_sixteen_levels():
    x = _rows(4, 9)
    codes, scale, zero = kq.quantize_rows(x)
    for r in range(x.shape[0]):
        for e in range(x.shape[1]):
            g = e // 32
            levels = float(zero[r, g]) + np.arange(16, dtype=np.float64) * float(scale[r, g])
            d = np.abs(levels - float(x[r, e]))
            assert d[codes[r, e]] <= d.min() + 1e-5 * float(scale[r, g])


def test_k4_rows_on_a_sixteen_level_grid_come_back_exactly():
    rng = np.random.default_rng(5)
    for step, lo in [(0.25, -1.0), (0.5, -4.0), (2.0 ** -6, 0.125), (8.0, -64.0)]:
        k = rng.integers(0, 16, size=(6, 128))
        k[:, 0::32] = 0          # every group spans the whole grid
        k[:, 1::32] = 15
        x = (lo + k * step).astype(np.float32)
        assert np.array_equal(_bf16(x), x)
        codes, scale, zero = kq.quantize_rows(x)
        assert np.array_equal(codes, k.astype(np.uint8))
        assert np.all(scale == np.float32(step)) and np.all(zero == np.float32(lo))
        assert np.array_equal(kq.dequantize_rows(codes, scale, zero), x)


def test_k5_constant_groups_min_and_max():
    x = _rows(6, 5)
    x[0, 32:64] = np.float32(0.75)               # constant group
    x[1, :] = np.float32(-3.0)                   # constant row
    codes, scale, zero = kq.quantize_rows(x)
    y = kq.dequantize_rows(codes, scale, zero)
    assert np.all(codes[0, 32:64] == 0) and scale[0, 1] == 0 and np.all(y[0, 32:64] == np.float32(0.75))
    assert np.all(codes[1] == 0) and np.all(y[1] == np.float32(-3.0))
    for r in range(2, 5):
        for g in range(4):
            grp = x[r, g * 32:(g + 1) * 32]
            c = codes[r, g * 32:(g + 1) * 32]
            assert c[np.argmin(grp)] == 0 and c[np.argmax(grp)] == 15
            assert y[r, g * 32 + np.argmin(grp)] == grp.min()      # the zero point is stored exactly


def test_k6_byte_layout_of_a_row_written_by_hand():
    # channel e carries code e % 16 on the grid -2 + 0.5 * code: scale 0.5 = bf16 0x3F00, zero -2 = bf16 0xC000
    x = (-2.0 + 0.5 * (np.arange(128) % 16)).astype(np.float32)[None, :]
    row = kq.pack_rows(*kq.quantize_rows(x))
    assert row.shape == (1, 80) and row.dtype == np.uint8
    codes_bytes = [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE] * 8
    want = bytes(codes_bytes) + bytes([0x00, 0x3F] * 4) + bytes([0x00, 0xC0] * 4)
    assert row.tobytes() == want
    codes, scale, zero = kq.unpack_rows(row)
    assert np.array_equal(codes[0], (np.arange(128) % 16).astype(np.uint8))
    assert np.all(scale == 0.5) and np.all(zero == -2.0)


def test_k7_pack_unpack_inverse():
    x = _rows(7, 11)
    codes, scale, zero = kq.quantize_rows(x)
    c2, s2, z2 = kq.unpack_rows(kq.pack_rows(codes, scale, zero))
    assert np.array_equal(c2, codes) and np.array_equal(s2, scale) and np.array_equal(z2, zero)


def test_k8_tiny_ranges_are_stored_as_constants_and_bad_inputs_rejected():
    x = np.zeros((1, 128), dtype=np.float32)
    x[0, :32] = np.float32(2.0 ** -126)
    x[0, 1] = np.float32(2.0 ** -125)
    codes, scale, zero = kq.quantize_rows(x)
    assert np.all(codes == 0) and np.all(scale == 0)
    with pytest.raises(ValueError):
        kq.quantize_rows(np.full((1, 128), 1.0 + 2.0 ** -12))


def _on_grid(seed, n):
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 16, size=(n, 128))
    k[:, 0::32] = 0
    k[:, 1::32] = 15
    return (-1.875 + 0.25 * k).astype(np.float32)


def test_k9_attention_over_on_grid_rows_equals_the_exact_oracle():
    """Quantisation is lossless for these rows, so Algorithm 1 over the 4-bit cache must give Eq. 3's values."""
    S, G, chunk = 45, 2, 16
    K, V = _on_grid(8, S), _on_grid(9, S)
    Q = _rows(10, G * S).reshape(G, S, 128)
    cache = kq.QuantizedHeadCache()
    got = kq.prefill_chunked_kv4(cache, Q, K, V, chunk)
    want = oa.attn_head(Q, K, V, 0)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    q, kn, vn = _rows(11, G), _on_grid(12, 1)[0], _on_grid(13, 1)[0]
    got = kq.decode_step_kv4(cache, q, kn, vn)
    Kall, Vall = np.concatenate([K, kn[None]]), np.concatenate([V, vn[None]])
    want = np.stack([oa.attn_rows(q[g][None].astype(np.float64), Kall, Vall, [S])[0] for g in range(G)])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    assert cache.length() == S + 1


def test_k10_one_chunk_sees_exact_rows_later_chunks_see_the_round_trip():
    S, G = 40, 2
    K, V = _rows(14, S), _rows(15, S)
    Q = _rows(16, G * S).reshape(G, S, 128)
    one = kq.prefill_chunked_kv4(kq.QuantizedHeadCache(), Q, K, V, S)
    np.testing.assert_allclose(one, oa.attn_head(Q, K, V, 0), rtol=0, atol=1e-12)
    # two chunks: rows 24.. attend to the round trip of rows 0..23 and to their own exact rows
    two = kq.prefill_chunked_kv4(kq.QuantizedHeadCache(), Q, K, V, 24)
    np.testing.assert_allclose(two[:, :24], one[:, :24], rtol=0, atol=1e-12)
    Kmix = np.concatenate([kq.roundtrip(K[:24]), K[24:]]).astype(np.float64)
    Vmix = np.concatenate([kq.roundtrip(V[:24]), V[24:]]).astype(np.float64)
    np.testing.assert_allclose(two[:, 24:], oa.attn_head(Q[:, 24:], Kmix, Vmix, 24), rtol=0, atol=1e-12)
    # and the approximation is a small perturbation of the exact result, not something else
    rel = np.linalg.norm(two - one) / np.linalg.norm(one)
    assert 0 < rel < 0.2


def test_k11_chunk_lengths_given_as_a_list():
    S, G = 50, 1
    K, V = _rows(17, S), _rows(18, S)
    Q = _rows(19, G * S).reshape(G, S, 128)
    a = kq.prefill_chunked_kv4(kq.QuantizedHeadCache(), Q, K, V, 20)
    b = kq.prefill_chunked_kv4(kq.QuantizedHeadCache(), Q, K, V, [20, 20, 10])
    assert np.array_equal(a, b)
    c = kq.prefill_chunked_kv4(kq.QuantizedHeadCache(), Q, K, V, [7, 43])
    Kmix = np.concatenate([kq.roundtrip(K[:7]), K[7:]]).astype(np.float64)
    Vmix = np.concatenate([kq.roundtrip(V[:7]), V[7:]]).astype(np.float64)
    np.testing.assert_allclose(c[:, 7:], oa.attn_head(Q[:, 7:], Kmix, Vmix, 7), rtol=0, atol=1e-12)
