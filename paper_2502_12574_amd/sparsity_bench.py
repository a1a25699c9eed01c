"""Head-wise sparsity (Appendix E, Table 14): one Llama-3-8B-shaped layer (8 KV heads, G = 4) with some of its
heads streaming (sink + recent tokens, bounded HBM store) and the others retrieval heads offloaded to pinned
host memory under a one-head HBM budget.

    python -m paper_2502_12574_amd.sparsity_bench [--context 1048576] [--chunk 16384] [--streaming 0,4]
                                                  [--sink 128] [--recent 512] [--decode-tokens 8]

Prints, per number of streaming heads, the wall time of the layer's chunked prefill (tokens/s per layer) and of a
decode token, plus the time spent in the streaming heads' own kernels.  The paper reports close to 2x for both
phases at 50 % sparsity (4 of 8 heads).  Inputs are random bf16 (timing only; parity is what
tests/test_gpu_streaming_heads.py checks).
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import binding as hb
from .session import Session

H, G, D = 8, 4, 128


def run(S, C, T, n_sink, n_recent, n_dec, stream_group, link_kv_bits=0):
    dev = "cuda:0"
    with Session(1, H, G, S + n_dec, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=0, streaming_heads=T, sink_tokens=n_sink,
                 recent_tokens=n_recent, link_kv_bits=link_kv_bits) as ss:
        gen = torch.Generator(device=dev).manual_seed(1)
        q = torch.randn(H, G, C, D, device=dev, generator=gen).to(torch.bfloat16)
        k = torch.randn(H, C, D, device=dev, generator=gen).to(torch.bfloat16)
        v = torch.randn(H, C, D, device=dev, generator=gen).to(torch.bfloat16)
        out = torch.empty(H, G, C, D, dtype=torch.bfloat16, device=dev)
        qd, kd, vd = q[:, :, 0].contiguous(), k[:, 0].contiguous(), v[:, 0].contiguous()
        outd = torch.empty(H, G, D, dtype=torch.bfloat16, device=dev)
        # calls of a layer: the retrieval heads one by one, then the streaming heads in groups
        calls = [(h, 1) for h in range(H - T)] + [(h, min(stream_group, H - h)) for h in range(H - T, H, stream_group)]
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
        if T > 0:
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
        stats = ss.stats()
    return dict(streaming_heads=T, link_kv_bits=link_kv_bits or 16, decode_h2d_MB_per_token=dec_h2d / 1e6,
                decode_link_GBps=dec_h2d / t_dec / 1e9, prefill_s=t_pre, prefill_tokens_per_s=S / t_pre, decode_ms_per_token=t_dec * 1e3,
                stream_prefill_kernels_s=t_stream_pre, stream_decode_kernels_us=t_stream_dec * 1e6,
                host_cache_GiB=ss.plan.host_bytes_total / 2**30, hbm_stream_MiB=ss.plan.hbm_stream_bytes / 2**20)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--context", type=int, default=1 << 20)
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--streaming", default="0,4")
    ap.add_argument("--sink", type=int, default=128)
    ap.add_argument("--recent", type=int, default=512)
    ap.add_argument("--decode-tokens", type=int, default=8)
    ap.add_argument("--stream-group", type=int, default=4, help="streaming heads per call")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("a GPU is required")
    rows = []
    for T in [int(x) for x in a.streaming.split(",")]:
        r = run(a.context, a.chunk, T, a.sink, a.recent, a.decode_tokens, max(1, a.stream_group))
        rows.append(r)
        print(json.dumps(r), flush=True)
    if len(rows) > 1 and rows[0]["streaming_heads"] == 0:
        for r in rows[1:]:
            print(f"streaming {r['streaming_heads']} of {H} heads (sink {a.sink}, recent {a.recent}): prefill "
                  f"{rows[0]['prefill_s'] / r['prefill_s']:.2f}x, decode "
                  f"{rows[0]['decode_ms_per_token'] / r['decode_ms_per_token']:.2f}x of the all-retrieval layer")


if __name__ == "__main__":
    main()
