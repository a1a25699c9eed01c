"""Pins of oracle/memory_model.py against the values the paper prints (tests/golden/paper_memory_tables.json)."""
import json
import os

import pytest

from oracle import memory_model as mm

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_memory_tables.json")))
M = mm.LLAMA3_8B


def _printed_close(value, printed, digits_tol=0.0051):
    """A printed table entry is the value rounded (or truncated) to the shown digits."""
    s = repr(printed)
    decimals = len(s.split(".")[1]) if "." in s and not s.endswith(".0") else 0
    unit = 10.0 ** (-decimals)
    return abs(value - printed) <= unit * 1.0001  # rounding or truncation to the printed digit


@pytest.mark.parametrize("method", ["standard", "chunked", "kv4bit", "layerwise", "headwise"])
def test_table10_rows(method):
    t = GOLD["table10_1M_context"]
    row = mm.memory_table_row(M, t["S"], method)
    for key, printed in t["rows"][method].items():
        assert _printed_close(row[key], printed), (method, key, row[key], printed)


@pytest.mark.parametrize("method", ["standard", "chunked", "kv4bit", "layerwise", "headwise"])
def test_table11_rows(method):
    g = GOLD["table11_max_context"]["rows"][method]
    S = g["S_K"] * 1024
    row = mm.memory_table_row(M, S, method)
    for key in ("kv", "activation", "total", "total_kv"):
        assert _printed_close(row[key], g[key]), (method, key, row[key], g[key])


def test_eq10_alpha_and_eq11_head_bytes():
    assert mm.alpha_headwise(M) == GOLD["alpha"]["value"] == 1 / 256
    # Eq. 11 at 1M tokens: 2 * 1 * 2^20 * 128 * 2 B = 512 MiB; two of them (ping-pong) are Table 10's "1" GB
    assert mm.head_bytes(M, 1 << 20) == 512 << 20
    assert mm.on_gpu_kv_bytes(M, 1 << 20, "headwise") == 1 << 30
    # Eq. 4-5: alpha times the whole cache is one head's bytes
    assert mm.alpha_headwise(M) * mm.kv_cache_bytes(M, 1 << 20) == mm.head_bytes(M, 1 << 20)


def _two_digits(value, printed):
    """Roofline table entries carry two or three significant digits."""
    return abs(value - printed) <= 0.06 * abs(printed)


def test_table12_prefill_counts():
    t = GOLD["table12_roofline_rtx4090"]
    for row in t["prefill"]:
        S = row["S_K"] * 1024
        one = row["heads"] == "one"
        ops = mm.prefill_ops(M, S, heads=4 if one else None)
        mem = mm.prefill_bytes_all(M, S, kv_heads=1 if one else None)
        kv = mm.prefill_bytes_kv(M, S, kv_heads=1 if one else None)
        assert _two_digits(ops, row["ops"]), row
        assert _two_digits(mem, row["mem"]), row
        assert _two_digits(kv, row["kv_mem"]), row
        assert _two_digits(ops / mem, row["intensity"]), row
        assert _two_digits(ops / kv, row["kv_intensity"]), row
        attain = mm.attainable_flops(ops / kv, t["peak_TFLOPs"] * 1e12, t["link_GBps"] * 1e9)
        bound = "memory" if attain < t["peak_TFLOPs"] * 1e12 else "compute"
        assert bound == row["offload_bound"], row
        if row["offload_flops"] is not None:
            assert _two_digits(attain, row["offload_flops"]), row


def test_table12_decode_ops():
    for row in GOLD["table12_roofline_rtx4090"]["decode_ops"]:
        S = row["S_K"] * 1024
        ops = mm.decode_ops(M, S, heads=4 if row["heads"] == "one" else None)
        assert _two_digits(ops, row["ops"]), row


def test_headwise_intensity_equals_full_attention():
    # Section 5: head-wise evaluation does not move the point on the roofline
    for S in (1024, 10240, 102400):
        a = mm.prefill_ops(M, S) / mm.prefill_bytes_kv(M, S)
        b = mm.prefill_ops(M, S, heads=4) / mm.prefill_bytes_kv(M, S, kv_heads=1)
        assert a == b


def test_causal_flops_closed_forms():
    # sum over chunks of the unit flops equals the layer closed form
    S, C, G, d = 4096, 512, 4, 128
    tot = sum(mm.causal_flops_unit(G, min(C, S - p), p, d) for p in range(0, S, C))
    assert tot * 8 == mm.causal_flops_layer(32, S, d)
    # brute-force pair count on a tiny case
    G, C, P = 2, 5, 7
    pairs = sum(1 for g in range(G) for i in range(C) for j in range(P + C) if j <= P + i)
    assert mm.causal_flops_unit(G, C, P, 8) == 4 * 8 * pairs
    h2d, d2h = mm.link_bytes_prefill_head(131072, 8192, 128)
    assert h2d == 480 << 20 and d2h == 64 << 20
