"""Head-group sweep: time one Llama-3-8B-shaped layer (8 KV heads, G = 4) with 1, 2, 4 or 8 KV heads per call.

    python -m paper_2502_12574_amd.group_bench [--contexts 1024,4096,...] [--decode-tokens 16] [--resident]

Section 4 ("adaptive head-wise offloading") fuses heads at shorter contexts because the per-head overheads
(launches, small transfers) dominate there; this prints, per context and group size, the wall time of the layer's
chunked prefill and of a decode token, K/V offloaded to pinned host memory with a one-head HBM budget (or resident
in HBM with --resident).  The library's plan reports the group size this sweep supports (hi_plan.heads_per_group).
Inputs are random bf16 (timing only; parity of grouped calls is what tests/test_gpu_head_groups.py checks).
"""
from __future__ import annotations

import argparse
import time

import torch

from . import binding as hb
from .session import Session

H, G, D = 8, 4, 128


def run(S, C, group, n_dec, mode, reps, resident_heads=0, decode_only=False):
    dev = "cuda:0"
    with Session(1, H, G, S + n_dec, C, mode=mode, out_fp32=0, gpu_kv_budget_heads=resident_heads + 1,
                 resident_heads=resident_heads) as ss:
        if mode == hb.HI_MODE_OFFLOAD and group * 64 > ss.plan.slice_tokens:
            return None
        gen = torch.Generator(device=dev).manual_seed(1)
        chunks = []
        for p in range(0, 0 if decode_only else S, C):
            n = min(C, S - p)
            chunks.append((p, n, torch.randn(H, G, n, D, device=dev, generator=gen).to(torch.bfloat16),
                           torch.randn(H, n, D, device=dev, generator=gen).to(torch.bfloat16),
                           torch.randn(H, n, D, device=dev, generator=gen).to(torch.bfloat16)))
        out = torch.empty(H, G, C, D, dtype=torch.bfloat16, device=dev)
        qd = torch.randn(H, G, D, device=dev, generator=gen).to(torch.bfloat16)
        kd = torch.randn(H, D, device=dev, generator=gen).to(torch.bfloat16)
        outd = torch.empty(H, G, D, dtype=torch.bfloat16, device=dev)
        units = [(ci, h0) for ci in range(len(chunks)) for h0 in range(0, H, group)]

        def prefill():
            with torch.cuda.stream(ss.s_compute):
                for u, (ci, h0) in enumerate(units):
                    p, n, q, k, v = chunks[ci]
                    nxt = None
                    if u + 1 < len(units):
                        nxt = (0, units[u + 1][1], group, chunks[units[u + 1][0]][0])
                    o = out[h0:h0 + group].view(-1)[:group * G * n * D].view(group, G, n, D)
                    ss.prefill_group(0, h0, group, q[h0:h0 + group], k[h0:h0 + group], v[h0:h0 + group], p, o, nxt)
            ss.sync()

        def decode():
            with torch.cuda.stream(ss.s_compute):
                for t in range(n_dec):
                    for h0 in range(0, H, group):
                        last = t + 1 == n_dec and h0 + group >= H
                        nxt = None if last else ((0, h0 + group, group, S + t) if h0 + group < H else (0, 0, group, S + t + 1))
                        ss.decode_group(0, h0, group, qd[h0:h0 + group], kd[h0:h0 + group], kd[h0:h0 + group], S + t,
                                        outd[h0:h0 + group], nxt)
            ss.sync()

        t_pre = float("nan")
        if not decode_only:
            prefill()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                prefill()
            t_pre = (time.perf_counter() - t0) / reps
        decode()
        t0 = time.perf_counter()
        for _ in range(reps):
            decode()
        t_dec = (time.perf_counter() - t0) / reps / n_dec
    return t_pre, t_dec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--contexts", default="1024,4096,16384,65536,262144")
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--decode-tokens", type=int, default=16)
    ap.add_argument("--resident", action="store_true")
    ap.add_argument("--resident-heads", default="", help="comma list: instead of the group sweep, keep that many of "
                    "the 8 KV heads in HBM (Algorithm 1's H_on, budget = that many + 1 heads), one head per call")
    ap.add_argument("--decode-only", action="store_true", help="skip the prefill timing (the cache content is "
                    "irrelevant to the decode timing)")
    args = ap.parse_args()
    mode = hb.HI_MODE_RESIDENT if args.resident else hb.HI_MODE_OFFLOAD
    print(f"one layer, {H} KV heads x G = {G}, chunk min(context, {args.chunk}), "
          f"{'HBM-resident' if args.resident else 'offloaded, one-head HBM budget'}; "
          "prefill ms per layer / decode ms per token per layer", flush=True)
    for S in [int(x) for x in args.contexts.split(",")]:
        C = min(S, args.chunk)
        reps = 20 if S <= 16384 else 5 if S <= 65536 else 2
        if args.resident_heads:
            for r in [int(x) for x in args.resident_heads.split(",")]:
                t_pre, t_dec = run(S, C, 1, args.decode_tokens, hb.HI_MODE_OFFLOAD, reps, r, args.decode_only)
                print(f"context {S:8d}: {r} of {H} heads in HBM: prefill {t_pre * 1e3:10.3f} ms per layer, "
                      f"decode {t_dec * 1e3:8.3f} ms per token per layer", flush=True)
            continue
        cells = []
        for group in (1, 2, 4, 8):
            r = run(S, C, group, args.decode_tokens, mode, reps)
            cells.append("      n/a      " if r is None else f"{r[0] * 1e3:8.3f} / {r[1] * 1e3:6.3f}")
        print(f"context {S:8d}: " + "  | ".join(f"group {g}: {c}" for g, c in zip((1, 2, 4, 8), cells)), flush=True)


if __name__ == "__main__":
    main()
