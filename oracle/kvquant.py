"""Oracle: 4-bit K/V rows on the far side of the host link, and head-wise attention over such a cache.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed.  Appendix B and Section 6.3 describe 4-bit KV quantisation as a representation that shrinks the
cache by about 4x (a uniform 4-bit code per element, converted back on the GPU before attention); the paper uses
it as a stand-alone baseline and names larger host tiers as future work.  Here it is composed with head-wise
offload: the rows of a head that leave HBM are stored as 4-bit codes, so the link (the bound of offloaded decode,
Section 3.3) carries about 3.2x fewer bytes; the rows of the chunk (or token) being processed are still the exact
bf16 ones, because they never crossed the link.  The paper fixes no code format; the reading taken:

  * per token row and per group of 32 consecutive channels: zero = min of the group, scale = (max - min) / 15,
    code = round-to-nearest-even((x - zero) / scale) clipped to [0, 15], x^ = zero + code * scale;
  * scale and zero are stored as bf16 (zero is a bf16 input value, so exact); a group whose scale rounds to less
    than 2^-120 is stored as the constant `zero` (all codes 0);
  * a row of 128 channels is 80 bytes on the link: 64 bytes of codes (channel 2i in the low nibble of byte i,
    channel 2i + 1 in the high nibble), 4 bf16 scales, 4 bf16 zeros (little endian).

Because floating point decides integers here (the codes), the steps are taken in the precision the kernel uses,
IEEE binary32 with one rounding per operation, in this order:
    s32   = fl32( fl32(max - min) * fl32(1/15) )          scale = bf16_rne(s32)
    inv   = fl32( 1 / scale )
    code  = min(15, rint( fl32( fl32(x - min) * inv ) ))
    x^    = bf16_rne( fl32( min + code * scale ) )         (code * scale is exact in binary32)
Inputs must be bf16-representable.  Attention over the cache is the exact fp64 definition (oracle/attention.py,
Eq. 3 and 7-9) applied to [x^ of the past rows ; exact rows of the current chunk], in Algorithm 1's order.

Pins (tests/test_oracle_kvquant.py): the reconstruction error bound in exact rational arithmetic; the chosen code
is the nearest of the 16 levels evaluated in fp64; inputs that lie on a 16-level grid are reproduced exactly;
constant groups; min -> code 0 and max -> code 15; the byte layout against a hand-written 80-byte row; attention
over a cache of on-grid rows equals the exact oracle; a prompt processed as one chunk equals the exact oracle
whatever the values (nothing has crossed the link yet).
"""
from __future__ import annotations

import numpy as np

from . import attention as oa

GROUP = 32
ROW_BYTES_128 = 80
_TINY = np.float32(2.0 ** -120)
_INV15 = np.float32(1.0) / np.float32(15.0)


def bf16_rne(x32: np.ndarray) -> np.ndarray:
    """Round binary32 values to the nearest bf16 (ties to even); result held in binary32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(np.shape(x32))


def _check_bf16(x: np.ndarray) -> np.ndarray:
    x32 = np.asarray(x, dtype=np.float32)
    if not np.array_equal(x32.astype(np.float64), np.asarray(x, dtype=np.float64)) or \
            np.any(x32.view(np.uint32) & 0xFFFF):
        raise ValueError("inputs must be bf16-representable")
    return x32


def quantize_rows(x):
    """x [n, d] (d a multiple of 32, bf16-representable).  Returns codes uint8 [n, d] in 0..15, scale and zero
    float32 [n, d / 32] holding bf16 values."""
    x32 = _check_bf16(x)
    n, d = x32.shape
    g = x32.reshape(n, d // GROUP, GROUP)
    mn = g.min(axis=2)
    mx = g.max(axis=2)
    s32 = (mx - mn).astype(np.float32) * _INV15
    scale = bf16_rne(s32.astype(np.float32))
    live = scale >= _TINY
    scale = np.where(live, scale, np.float32(0.0)).astype(np.float32)
    inv = np.zeros_like(scale)
    inv[live] = np.float32(1.0) / scale[live]
    t = ((g - mn[:, :, None]).astype(np.float32) * inv[:, :, None]).astype(np.float32)
    codes = np.minimum(np.rint(t), np.float32(15.0)).astype(np.uint8)
    return codes.reshape(n, d), scale, mn.astype(np.float32)


def dequantize_rows(codes, scale, zero) -> np.ndarray:
    """Inverse map; returns float32 [n, d] holding bf16 values."""
    codes = np.asarray(codes)
    n, d = codes.shape
    c = codes.reshape(n, d // GROUP, GROUP).astype(np.float32)
    prod = (c * np.asarray(scale, np.float32)[:, :, None]).astype(np.float32)          # exact: 4 bits x 8 bits
    y32 = (np.asarray(zero, np.float32)[:, :, None] + prod).astype(np.float32)
    return bf16_rne(y32).reshape(n, d)


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def pack_rows(codes, scale, zero) -> np.ndarray:
    """The link representation: uint8 [n, d/2 + 4 * (d/32)] (80 bytes for d = 128)."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, d = codes.shape
    nib = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    s = _bf16_bits(scale).astype("<u2").view(np.uint8).reshape(n, -1)
    z = _bf16_bits(zero).astype("<u2").view(np.uint8).reshape(n, -1)
    return np.concatenate([nib, s, z], axis=1)


def unpack_rows(rows: np.ndarray, d: int = 128):
    rows = np.asarray(rows, dtype=np.uint8)
    n = rows.shape[0]
    ng = d // GROUP
    nib = rows[:, :d // 2]
    codes = np.empty((n, d), dtype=np.uint8)
    codes[:, 0::2] = nib & 15
    codes[:, 1::2] = nib >> 4
    def bf(b):
        u = np.ascontiguousarray(b).view("<u2").astype(np.uint32) << 16
        return u.view(np.float32).reshape(n, ng)
    return codes, bf(rows[:, d // 2:d // 2 + 2 * ng]), bf(rows[:, d // 2 + 2 * ng:d // 2 + 4 * ng])


def roundtrip(x) -> np.ndarray:
    """What the GPU sees of rows that went to the host and came back."""
    return dequantize_rows(*quantize_rows(x))


class QuantizedHeadCache:
    """The host-side history of one (layer, KV head): packed rows, K and V."""

    def __init__(self, head_dim: int = 128):
        self.d = head_dim
        w = head_dim // 2 + 4 * (head_dim // GROUP)
        self.K = np.zeros((0, w), dtype=np.uint8)
        self.V = np.zeros((0, w), dtype=np.uint8)

    def length(self) -> int:
        return self.K.shape[0]

    def history(self):
        """Dequantised K and V of everything stored, float64."""
        k = dequantize_rows(*unpack_rows(self.K, self.d)).astype(np.float64)
        v = dequantize_rows(*unpack_rows(self.V, self.d)).astype(np.float64)
        return k, v

    def append(self, k_rows, v_rows):
        self.K = np.concatenate([self.K, pack_rows(*quantize_rows(k_rows))], axis=0)
        self.V = np.concatenate([self.V, pack_rows(*quantize_rows(v_rows))], axis=0)


def prefill_chunked_kv4(cache: QuantizedHeadCache, Q, K, V, chunk) -> np.ndarray:
    """Algorithm 1's prefill for one KV head with a 4-bit host cache.  Q [G, S, d]; K, V [S, d]; chunk: the chunk
    length, or the list of the chunks' lengths (summing to S).  Per chunk: attend to [dequantised past ; the chunk's
    exact rows] (Eq. 3 with the causal mask), then the chunk's rows go to the cache.  Returns [G, S, d] float64."""
    Q = np.asarray(Q, dtype=np.float64)
    K32, V32 = _check_bf16(K), _check_bf16(V)
    S = K32.shape[0]
    out = np.empty_like(Q)
    lengths = [chunk] * (-(-S // chunk)) if isinstance(chunk, (int, np.integer)) else list(chunk)
    starts = np.concatenate([[0], np.cumsum(lengths)])[:len(lengths)]
    for c0, n in zip(starts, lengths):
        c0 = int(c0)
        c1 = min(S, c0 + int(n))
        past = cache.length()
        kp, vp = cache.history()
        Kh = np.concatenate([kp, K32[c0:c1].astype(np.float64)], axis=0)
        Vh = np.concatenate([vp, V32[c0:c1].astype(np.float64)], axis=0)
        out[:, c0:c1] = oa.attn_head(Q[:, c0:c1], Kh, Vh, past)
        cache.append(K32[c0:c1], V32[c0:c1])
    return out


def decode_step_kv4(cache: QuantizedHeadCache, q, k_new, v_new) -> np.ndarray:
    """One token of one KV head: q [G, d]; k_new, v_new [d].  The token attends to the dequantised past and to
    its own exact row, which then goes to the cache.  Returns [G, d] float64."""
    q = np.asarray(q, dtype=np.float64)
    k32, v32 = _check_bf16(k_new)[None, :], _check_bf16(v_new)[None, :]
    kp, vp = cache.history()
    Kh = np.concatenate([kp, k32.astype(np.float64)], axis=0)
    Vh = np.concatenate([vp, v32.astype(np.float64)], axis=0)
    p = Kh.shape[0] - 1
    out = np.stack([oa.attn_rows(q[g][None, :], Kh, Vh, [p])[0] for g in range(q.shape[0])])
    cache.append(k32, v32)
    return out
