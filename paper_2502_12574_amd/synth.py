"""Seeded synthetic inputs for the head-wise attention path.

This module only *draws inputs*: it holds none of the method's arithmetic (no scores, no softmax,
no memory model).  It serves the tests, the benchmark and the CPU oracle's callers alike, so that both
sides of a parity check see the same bits.

The paper evaluates on long-document benchmarks with a trained Llama-3-8B (Section 6); attention cost and
numerics depend only on tensor shapes and value scale, so post-RoPE Q/K/V are drawn directly as bf16
N(0,1) at Llama-3-8B shapes (32 query heads, 8 KV heads, head_dim 128).

Every element is a pure function of (seed, tensor, layer, head, token, dim), built from integer operations
only, so any row can be regenerated bit-exactly on the CPU or on the GPU, in any order and in slices:

    value = TABLE[ mix(seed, tensor, layer, head, token, dim) >> 16 ]

with TABLE[i] = bf16( Phi^-1((i + 1/2) / 65536) ), the 65 536-point quantile grid of the standard normal.
All integer arithmetic is done on values below 2**32 held in int64 with multipliers below 2**31, so no
product ever overflows a signed 64-bit integer and the CPU and GPU results agree bit for bit.
"""
from __future__ import annotations

import functools

import numpy as np
import torch

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_SCALE = 1, 2, 3, 4
TENSOR_X, TENSOR_WQKV, TENSOR_WO = 5, 6, 7

_M32 = 0xFFFFFFFF
# odd multipliers below 2**31 (so a 32-bit value times one of them stays below 2**63)
_MUL_A = 0x5F356495
_MUL_B = 0x32C446BD
_MUL_C = 0x6A09E667
_MUL_D = 0x3C6EF372 | 1


def _mix_int(x: int) -> int:
    """Scalar form of the avalanche step (Python ints), identical to `_mix_tensor`."""
    x &= _M32
    x ^= x >> 15
    x = (x * _MUL_A) & _M32
    x ^= x >> 13
    x = (x * _MUL_B) & _M32
    x ^= x >> 16
    return x


def _mix_tensor(x: torch.Tensor) -> torch.Tensor:
    """xorshift-multiply avalanche on int64 tensors whose values lie in [0, 2**32)."""
    x = x ^ (x >> 15)
    x = (x * _MUL_A) & _M32
    x = x ^ (x >> 13)
    x = (x * _MUL_B) & _M32
    x = x ^ (x >> 16)
    return x


def _stream_key(seed: int, tensor: int, layer: int, head: int) -> int:
    k = _mix_int(seed ^ 0x9E3779B9)
    k = _mix_int(k + tensor * _MUL_C)
    k = _mix_int(k + layer * _MUL_D)
    k = _mix_int(k + head * _MUL_A)
    return k


@functools.lru_cache(maxsize=None)
def _table_cpu() -> torch.Tensor:
    """bf16 standard-normal quantiles at the 65 536 mid-points (i + 1/2) / 65536."""
    from scipy.special import ndtri

    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    z = ndtri(p)
    return torch.from_numpy(z).to(torch.float32).to(torch.bfloat16)


_table_dev: dict = {}


def normal_table(device="cpu") -> torch.Tensor:
    dev = torch.device(device)
    if dev.type == "cpu":
        return _table_cpu()
    key = (dev.type, dev.index)
    if key not in _table_dev:
        _table_dev[key] = _table_cpu().to(dev)
    return _table_dev[key]


def token_hash(seed: int, tensor: int, layer: int, head: int, tok_start: int, n_tok: int,
               device="cpu") -> torch.Tensor:
    """32-bit hash of each token index in [tok_start, tok_start + n_tok), as int64."""
    key = _stream_key(seed, tensor, layer, head)
    tok = torch.arange(tok_start, tok_start + n_tok, dtype=torch.int64, device=device)
    lo = tok & _M32
    hi = (tok >> 32) & _M32          # contexts beyond 2**32 tokens are not expected, but stay defined
    return _mix_tensor(_mix_tensor(lo ^ key) + hi * 0x2545F491 & _M32)


def draw(seed: int, tensor: int, layer: int, head: int, tok_start: int, n_tok: int, head_dim: int = 128,
         device="cpu") -> torch.Tensor:
    """bf16 N(0,1) rows [n_tok, head_dim] of one tensor (Q, K or V) of one head."""
    if n_tok == 0:
        return torch.empty((0, head_dim), dtype=torch.bfloat16, device=device)
    th = token_hash(seed, tensor, layer, head, tok_start, n_tok, device)           # [n]
    dim = torch.arange(head_dim, dtype=torch.int64, device=device) * _MUL_C & _M32  # [d]
    x = _mix_tensor((th[:, None] + dim[None, :]) & _M32)
    return normal_table(device)[x >> 16]


def peaked_key_mask(seed: int, layer: int, head: int, tok_start: int, n_tok: int, device="cpu",
                    one_in: int = 10) -> torch.Tensor:
    """Boolean [n_tok]: which key rows are scaled up to make peaked softmax rows (about one in ten)."""
    th = token_hash(seed, TENSOR_SCALE, layer, head, tok_start, n_tok, device)
    return (th % one_in) == 0


def draw_keys_peaked(seed: int, layer: int, head: int, tok_start: int, n_tok: int, head_dim: int = 128,
                     device="cpu", factor: float = 4.0) -> torch.Tensor:
    """K rows with the selected rows multiplied by a power of two (exact in bf16)."""
    k = draw(seed, TENSOR_K, layer, head, tok_start, n_tok, head_dim, device)
    m = peaked_key_mask(seed, layer, head, tok_start, n_tok, device)
    scale = torch.where(m, factor, 1.0).to(torch.float32)
    return (k.to(torch.float32) * scale[:, None]).to(torch.bfloat16)


def draw_q(seed, layer, q_head, tok_start, n_tok, head_dim=128, device="cpu", scale=1.0):
    """scale != 1: the drawn rows times `scale`, multiplied in fp32 and rounded to bf16 (queries as a projection
    that folds a constant into them would emit them)."""
    q = draw(seed, TENSOR_Q, layer, q_head, tok_start, n_tok, head_dim, device)
    if scale == 1.0:
        return q
    return (q.to(torch.float32) * torch.tensor(scale, dtype=torch.float32, device=q.device)).to(torch.bfloat16)


def draw_k(seed, layer, kv_head, tok_start, n_tok, head_dim=128, device="cpu", peaked=False):
    if peaked:
        return draw_keys_peaked(seed, layer, kv_head, tok_start, n_tok, head_dim, device)
    return draw(seed, TENSOR_K, layer, kv_head, tok_start, n_tok, head_dim, device)


def draw_v(seed, layer, kv_head, tok_start, n_tok, head_dim=128, device="cpu"):
    return draw(seed, TENSOR_V, layer, kv_head, tok_start, n_tok, head_dim, device)


def draw_hidden(seed, layer, tok_start, n_tok, d_model, device="cpu"):
    """bf16 N(0,1) hidden states [n_tok, d_model] entering a layer's attention block."""
    return draw(seed, TENSOR_X, layer, 0, tok_start, n_tok, d_model, device)


def draw_weight(seed, tensor, layer, out_features, in_features, device="cpu"):
    """bf16 weight [out_features, in_features] (the layout of y = x W^T): N(0,1) scaled by the power of two nearest
    to 1/sqrt(in_features) (exact in bf16), so that projections of N(0,1) rows come out near unit variance."""
    import math

    w = draw(seed, tensor, layer, 0, 0, out_features, in_features, device)
    scale = 2.0 ** (-round(math.log2(in_features) / 2.0))
    return (w.to(torch.float32) * scale).to(torch.bfloat16)


def to_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of a bf16/fp32 tensor to a float64 numpy array on the host."""
    return x.detach().to("cpu").to(torch.float64).numpy()
