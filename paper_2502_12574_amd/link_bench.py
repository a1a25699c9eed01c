"""4-bit rows on the host link against bf16 rows: one Llama-3-8B-shaped layer (8 KV heads, G = 4), every head
offloaded to pinned host memory under a one-head HBM budget.

    python -m paper_2502_12574_amd.link_bench [--context 1048576] [--chunk 16384] [--decode-tokens 8]
                                              [--streaming 0] [--sink 128] [--recent 512]

Prints, per link format, the wall time of the layer's chunked prefill and of a decode token, and the bytes a decode
token moves over the link.  Offloaded decode is bound by the link (Section 3.3), so its time should follow the bytes
per row (512 -> 160 for K and V together); prefill is bound by the matrix pipes at this chunk size and should not
change.  --streaming T makes the last T heads streaming heads (Appendix E) in both runs, to see the two
reductions of link traffic composed.  Inputs are random bf16 (timing only; parity is what tests/test_gpu_kvquant.py checks).
"""
from __future__ import annotations

import argparse
import json

import torch

from .sparsity_bench import run


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--context", type=int, default=1 << 20)
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--decode-tokens", type=int, default=8)
    ap.add_argument("--bits", default="16,4")
    ap.add_argument("--streaming", type=int, default=0)
    ap.add_argument("--sink", type=int, default=128)
    ap.add_argument("--recent", type=int, default=512)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("a GPU is required")
    rows = []
    for bits in [int(x) for x in a.bits.split(",")]:
        r = run(a.context, a.chunk, a.streaming, a.sink if a.streaming else 0, a.recent if a.streaming else 0,
                a.decode_tokens, max(1, a.streaming), link_kv_bits=0 if bits == 16 else bits)
        rows.append(r)
        print(json.dumps(r), flush=True)
    if len(rows) == 2:
        print(f"{rows[1]['link_kv_bits']}-bit rows against {rows[0]['link_kv_bits']}-bit rows: prefill "
              f"{rows[0]['prefill_s'] / rows[1]['prefill_s']:.2f}x, decode "
              f"{rows[0]['decode_ms_per_token'] / rows[1]['decode_ms_per_token']:.2f}x, host cache "
              f"{rows[0]['host_cache_GiB'] / rows[1]['host_cache_GiB']:.2f}x smaller")


if __name__ == "__main__":
    main()
