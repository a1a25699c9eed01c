"""fp64/integer oracle for the paper's memory and roofline arithmetic (what `hi_offload_plan` must reproduce).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Follows Eq. 4-6 (KV-cache size and on-GPU fraction), Eq. 10-11 (head-wise fraction and on-GPU bytes),
Appendix A.3 (per-method memory estimates behind Tables 10 and 11), Section 5 (T ~ max(T_comp, T_mem)) and
Appendix D (operation and byte counts behind Tables 12-13).

Readings taken (the tables only close with them): the symbol H is the number of KV heads per layer (8 for
Llama-3-8B) and D = H * D_h = 1024 is the KV width; "1K" = 1024 tokens, "GB" = 2**30 bytes; the roofline
tables count 4*S^2*d flops per query head (both contractions, no causal halving) and, for decode, the K/V
bytes of all query heads (no GQA sharing).

Pins (tests/test_oracle_memory_model.py): every value the paper prints in Tables 10, 11 and 12 for the
quantities modelled here, stored with citations under tests/golden/.
"""
from __future__ import annotations

from dataclasses import dataclass

GiB = float(2 ** 30)


@dataclass(frozen=True)
class ModelShape:
    n_layers: int = 32          # L
    n_q_heads: int = 32
    n_kv_heads: int = 8         # H (KV heads per layer)
    head_dim: int = 128         # D_h
    hidden: int = 4096          # model width (activations)
    intermediate: int = 14336   # I (MLP)
    dtype_bytes: int = 2
    weights_gib: float = 15.08  # as printed in Tables 10-11

    @property
    def kv_width(self) -> int:  # D = H * D_h
        return self.n_kv_heads * self.head_dim


LLAMA3_8B = ModelShape()


def kv_cache_bytes(m: ModelShape, S: int, batch: int = 1) -> int:
    """Eq. 4: 2 * B * L * S * D * sizeof."""
    return 2 * batch * m.n_layers * S * m.kv_width * m.dtype_bytes


def alpha_headwise(m: ModelShape, heads_on_gpu: int = 1) -> float:
    """Eq. 10: fraction of the cache on the GPU, H_on / (L * H)."""
    return heads_on_gpu / (m.n_layers * m.n_kv_heads)


def head_bytes(m: ModelShape, S: int, batch: int = 1) -> int:
    """Eq. 11: one head's K and V: 2 * B * S * D_h * sizeof."""
    return 2 * batch * S * m.head_dim * m.dtype_bytes


def on_gpu_kv_bytes(m: ModelShape, S: int, method: str, batch: int = 1) -> float:
    """GPU-side KV bytes of each method of Appendix A.3 (ping-pong methods hold two units)."""
    total = kv_cache_bytes(m, S, batch)
    if method in ("standard", "chunked"):
        return total
    if method == "kv4bit":
        return total / 4
    if method == "layerwise":
        return 2 * total / m.n_layers
    if method == "headwise":
        return 2 * head_bytes(m, S, batch)
    raise ValueError(method)


def activation_bytes(m: ModelShape, rows: int) -> int:
    """Appendix A.3: rows * D + 2 * rows * I elements."""
    return rows * (m.hidden + 2 * m.intermediate) * m.dtype_bytes


def memory_table_row(m: ModelShape, S: int, method: str, chunk: int = 10 * 1024) -> dict:
    """One row of Tables 10/11, in GiB: weights, GPU KV, activation, total, total KV across GPU and CPU."""
    act_rows = chunk if method in ("chunked", "headwise") else S
    kv = on_gpu_kv_bytes(m, S, method) / GiB
    act = activation_bytes(m, act_rows) / GiB
    total_kv = kv_cache_bytes(m, S) / GiB / (4 if method == "kv4bit" else 1)
    return {"weights": m.weights_gib, "kv": kv, "activation": act, "total": m.weights_gib + kv + act,
            "total_kv": total_kv}


# ---- Section 5 / Appendix D: operation and byte counts -------------------------------------------------

def prefill_ops(m: ModelShape, S: int, heads: int | None = None) -> float:
    """Tables 12-13 'Ops' for prefill: 4 * S^2 * d per query head (no causal halving)."""
    hq = m.n_q_heads if heads is None else heads
    return 4.0 * S * S * m.head_dim * hq


def prefill_bytes_all(m: ModelShape, S: int, kv_heads: int | None = None) -> float:
    """'Memory' (regular): Q, K, V and O bytes."""
    hk = m.n_kv_heads if kv_heads is None else kv_heads
    hq = hk * (m.n_q_heads // m.n_kv_heads)
    return float(2 * S * hq * m.head_dim * m.dtype_bytes + 2 * S * hk * m.head_dim * m.dtype_bytes)


def prefill_bytes_kv(m: ModelShape, S: int, kv_heads: int | None = None) -> float:
    """'Memory (KV cache)' (offload): only K and V cross the host link."""
    hk = m.n_kv_heads if kv_heads is None else kv_heads
    return float(2 * S * hk * m.head_dim * m.dtype_bytes)


def decode_ops(m: ModelShape, S: int, heads: int | None = None) -> float:
    hq = m.n_q_heads if heads is None else heads
    return 4.0 * S * m.head_dim * hq


def attainable_flops(intensity: float, peak_flops: float, bandwidth: float) -> float:
    """Roofline: min(peak, intensity * bandwidth); T ~ max(T_comp, T_mem) (Section 5)."""
    return min(peak_flops, intensity * bandwidth)


# ---- exact work of the causal head-wise evaluation (used for throughput accounting) ---------------------

def causal_flops_unit(G: int, C: int, P: int, d: int) -> int:
    """Useful flops of one prefill unit (chunk of C rows at past length P, one KV head, its G query heads):
    two contractions of 2*d flops per (query row, visible key) pair."""
    pairs = G * (C * P + C * (C + 1) // 2)
    return 4 * d * pairs


def causal_flops_layer(Hq: int, S: int, d: int) -> int:
    return 4 * d * Hq * (S * (S + 1) // 2)


def link_bytes_prefill_head(S: int, C: int, d: int, dtype_bytes: int = 2) -> tuple[int, int]:
    """(H2D, D2H) bytes of one KV head over a chunked prefill in Algorithm 1's loop order: before chunk c the
    head's past rows [0, c*C) come up, after it the chunk's rows go down."""
    row = 2 * d * dtype_bytes
    h2d = sum(min(p, S) * row for p in range(0, S, C))
    return h2d, S * row
