"""Wall-time measurements of one Llama-3-8B-shaped layer (8 KV heads, G = 4) under the head kinds and call shapes
the library offers, K/V offloaded to pinned host memory under a one-head HBM budget unless stated.

    python -m paper_2502_12574_amd.layer_bench [--context 1048576] [--chunk 16384] [--decode-tokens 8]
        [--streaming 0,4] [--sink 128] [--recent 512] [--stream-group 4]     head-wise sparsity (Appendix E, Table 14)
        [--link-bits 16,4]                                                     4-bit rows on the host link
        [--heads-per-call 1,2,4,8]                                             head groups (Section 4)
        [--resident-heads 0,4,7]                                               Algorithm 1's H_on (budget = that many + 1)
        [--resident]                                                           everything in HBM (no link)
        [--decode-only]                                                        skip the prefill timing

Every comma list is swept (the cross product, outermost first in the order above); one JSON line per run with the
wall time of the layer's chunked prefill and of a decode token, the link bytes a decode token moves and, for
streaming heads, the time of their own kernels.  Inputs are random bf16 (timing only; parity is what tests/ checks).
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import binding as hb
from .session import Session

H, G, D = 8, 4, 128


def run(S, C, T=0, n_sink=0, n_recent=0, n_dec=8, stream_group=1, link_kv_bits=0, heads_per_call=1, resident_heads=0,
        mode=hb.HI_MODE_OFFLOAD, decode_only=False, q_prescaled=False):
    """One layer: T streaming heads (the last T), the others retrieval heads called heads_per_call at a time."""
    dev = "cuda:0"
    with Session(1, H, G, S + n_dec, C, mode=mode, out_fp32=0, streaming_heads=T, sink_tokens=n_sink,
                 recent_tokens=n_recent, link_kv_bits=link_kv_bits, gpu_kv_budget_heads=resident_heads + 1,
                 resident_heads=resident_heads, q_prescaled=q_prescaled) as ss:
        if mode == hb.HI_MODE_OFFLOAD and heads_per_call * 64 > ss.plan.slice_tokens:
            return None                 # a staging slice cannot hold 64 rows of every head of the group
        gen = torch.Generator(device=dev).manual_seed(1)
        q = (torch.randn(H, G, C, D, device=dev, generator=gen) * (hb.HI_Q_PRESCALE if q_prescaled else 1.0)).to(torch.bfloat16)
        k = torch.randn(H, C, D, device=dev, generator=gen).to(torch.bfloat16)
        v = torch.randn(H, C, D, device=dev, generator=gen).to(torch.bfloat16)
        out = torch.empty(H, G, C, D, dtype=torch.bfloat16, device=dev)
        qd, kd, vd = q[:, :, 0].contiguous(), k[:, 0].contiguous(), v[:, 0].contiguous()
        outd = torch.empty(H, G, D, dtype=torch.bfloat16, device=dev)
        # calls of a layer: the retrieval heads in groups (never mixing HBM-resident and offloaded ones), then the
        # streaming heads in groups
        calls = []
        h = 0
        while h < H - T:
            lim = resident_heads if h < resident_heads else H - T
            calls.append((h, min(heads_per_call, lim - h)))
            h += calls[-1][1]
        calls += [(h, min(stream_group, H - h)) for h in range(H - T, H, stream_group)]
        starts = list(range(0, S, C))

        def nxt_of(ci, j, pasts):
            if j + 1 < len(calls):
                return (0, calls[j + 1][0], calls[j + 1][1], pasts[ci])
            if ci + 1 < len(pasts):
                return (0, calls[0][0], calls[0][1], pasts[ci + 1])
            return None

        def prefill():
            with torch.cuda.stream(ss.s_compute):
                for ci, p in enumerate(starts):
                    n = min(C, S - p)
                    for j, (h0, nh) in enumerate(calls):
                        o = out[h0:h0 + nh].view(-1)[:nh * G * n * D].view(nh, G, n, D)
                        ss.prefill_group(0, h0, nh, q[h0:h0 + nh, :, :n].contiguous() if n < C else q[h0:h0 + nh],
                                         k[h0:h0 + nh, :n].contiguous() if n < C else k[h0:h0 + nh],
                                         v[h0:h0 + nh, :n].contiguous() if n < C else v[h0:h0 + nh], p, o,
                                         nxt_of(ci, j, starts))
            ss.sync()

        def decode():
            pasts = [S + t for t in range(n_dec)]
            with torch.cuda.stream(ss.s_compute):
                for ti, p in enumerate(pasts):
                    for j, (h0, nh) in enumerate(calls):
                        ss.decode_group(0, h0, nh, qd[h0:h0 + nh], kd[h0:h0 + nh], vd[h0:h0 + nh], p, outd[h0:h0 + nh],
                                        nxt_of(ti, j, pasts))
            ss.sync()

        t_pre = float("nan")
        if not decode_only:
            prefill()                       # fills the cache and the stores; warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            prefill()
            t_pre = time.perf_counter() - t0
        decode()
        hb.hi_reset_stats(ss.ctx)
        t0 = time.perf_counter()
        decode()
        t_dec = (time.perf_counter() - t0) / n_dec
        dec_h2d = ss.stats().bytes_h2d / n_dec

        # the streaming heads' kernels alone (HIP events inside the library)
        t_stream_pre = t_stream_dec = 0.0
        if T > 0 and not decode_only:
            hb.hi_ctx_set_flags(ss.ctx, hb.HI_FLAG_TIME_KERNELS)
            hb.hi_reset_stats(ss.ctx)
            with torch.cuda.stream(ss.s_compute):
                for p in starts:
                    for h0, nh in calls:
                        if h0 >= H - T:
                            ss.prefill_group(0, h0, nh, q[h0:h0 + nh], k[h0:h0 + nh], v[h0:h0 + nh], p, out[h0:h0 + nh])
            ss.sync()
            t_stream_pre = ss.stats().prefill_kernel_ms * 1e-3
            hb.hi_reset_stats(ss.ctx)
            with torch.cuda.stream(ss.s_compute):
                for h0, nh in calls:
                    if h0 >= H - T:
                        ss.decode_group(0, h0, nh, qd[h0:h0 + nh], kd[h0:h0 + nh], vd[h0:h0 + nh], S, outd[h0:h0 + nh])
            ss.sync()
            t_stream_dec = ss.stats().decode_kernel_ms * 1e-3
            hb.hi_ctx_set_flags(ss.ctx, 0)
        host_gib, stream_mib = ss.plan.host_bytes_total / 2**30, ss.plan.hbm_stream_bytes / 2**20
    return dict(context=S, chunk=C, streaming_heads=T, link_kv_bits=link_kv_bits or 16, heads_per_call=heads_per_call,
                resident_heads=resident_heads, resident_mode=mode == hb.HI_MODE_RESIDENT,
                decode_h2d_MB_per_token=dec_h2d / 1e6, decode_link_GBps=dec_h2d / t_dec / 1e9, prefill_s=t_pre,
                prefill_tokens_per_s=S / t_pre, decode_ms_per_token=t_dec * 1e3, stream_prefill_kernels_s=t_stream_pre,
                stream_decode_kernels_us=t_stream_dec * 1e6, host_cache_GiB=host_gib, hbm_stream_MiB=stream_mib)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--context", default=str(1 << 20), help="comma list of context lengths")
    ap.add_argument("--chunk", type=int, default=16384, help="chunk = min(context, this)")
    ap.add_argument("--streaming", default="0")
    ap.add_argument("--sink", type=int, default=128)
    ap.add_argument("--recent", type=int, default=512)
    ap.add_argument("--decode-tokens", type=int, default=8)
    ap.add_argument("--stream-group", type=int, default=4, help="streaming heads per call")
    ap.add_argument("--link-bits", default="16")
    ap.add_argument("--heads-per-call", default="1")
    ap.add_argument("--resident-heads", default="0")
    ap.add_argument("--resident", action="store_true")
    ap.add_argument("--decode-only", action="store_true")
    ap.add_argument("--q-prescaled", action="store_true", help="queries that carry the softmax scale")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("a GPU is required")
    ints = lambda s: [int(x) for x in s.split(",")]
    mode = hb.HI_MODE_RESIDENT if a.resident else hb.HI_MODE_OFFLOAD
    rows = []
    for S in ints(a.context):
        for T in ints(a.streaming):
            for bits in ints(a.link_bits):
                for hpc in ints(a.heads_per_call):
                    for rh in ints(a.resident_heads):
                        r = run(S, min(S, a.chunk), T, a.sink if T else 0, a.recent if T else 0, a.decode_tokens,
                                max(1, a.stream_group), 0 if bits == 16 else bits, hpc, rh, mode, a.decode_only,
                                a.q_prescaled)
                        if r is None:
                            print(json.dumps(dict(context=S, heads_per_call=hpc, skipped="slice too short")), flush=True)
                            continue
                        rows.append(r)
                        print(json.dumps(r), flush=True)
    base = rows[0] if rows else None
    for r in rows[1:]:
        if r["context"] == base["context"]:
            print(f"streaming {r['streaming_heads']}, {r['link_kv_bits']}-bit link rows, {r['heads_per_call']} heads per call, "
                  f"{r['resident_heads']} resident: prefill {base['prefill_s'] / r['prefill_s']:.2f}x, decode "
                  f"{base['decode_ms_per_token'] / r['decode_ms_per_token']:.2f}x of the first run")


if __name__ == "__main__":
    main()
