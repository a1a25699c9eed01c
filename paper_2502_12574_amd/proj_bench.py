"""Projection micro-benchmark: the Q/K/V projection with rotary embedding (hi_qkv_rope) and the output projection
(hi_out_proj) of one chunk at Llama-3-8B shapes (d_model 4096, 32 query / 8 KV heads), HIP-event timed.

    python -m paper_2502_12574_amd.proj_bench [--chunk 16384] [--reps 10] [--past 1032192]

Algorithmic flops: 2 * chunk * d_model * (Hq + 2 Hkv) * 128 and 2 * chunk * (Hq * 128) * d_model.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as hb


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--past", type=int, default=(1 << 20) - 16384)
    ap.add_argument("--d-model", type=int, default=4096)
    ap.add_argument("--q-heads", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("a GPU is required")
    dev, C, D, Hq, Hkv = "cuda:0", a.chunk, a.d_model, a.q_heads, a.kv_heads
    gen = torch.Generator(device=dev).manual_seed(1)
    x = torch.randn(C, D, device=dev, generator=gen).to(torch.bfloat16)
    w = (torch.randn((Hq + 2 * Hkv) * 128, D, device=dev, generator=gen) / 64).to(torch.bfloat16)
    wo = (torch.randn(D, Hq * 128, device=dev, generator=gen) / 64).to(torch.bfloat16)
    q = torch.empty(Hq, C, 128, dtype=torch.bfloat16, device=dev)
    k = torch.empty(Hkv, C, 128, dtype=torch.bfloat16, device=dev)
    v = torch.empty(Hkv, C, 128, dtype=torch.bfloat16, device=dev)
    y = torch.empty(C, D, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(hb.hi_proj_workspace_bytes(C), dtype=torch.uint8, device=dev)
    s = torch.cuda.current_stream()

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(a.reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / a.reps * 1e-3

    t1 = timed(lambda: hb.hi_qkv_rope(s, x, w, D, Hq, Hkv, C, a.past, 500000.0, 0, q, k, v, ws))
    f1 = 2.0 * C * D * (Hq + 2 * Hkv) * 128
    print(f"qkv+rope  C={C}: {t1 * 1e3:.3f} ms, {f1 / t1 / 1e12:.1f} TFLOP/s ({f1 / t1 / 2.5e15 * 100:.1f}% of 2.5 PFLOP/s); "
          f"algorithmic flops {f1:.3e}", flush=True)
    t2 = timed(lambda: hb.hi_out_proj(s, q, wo, Hq, D, C, 0, y))
    f2 = 2.0 * C * Hq * 128 * D
    print(f"out_proj  C={C}: {t2 * 1e3:.3f} ms, {f2 / t2 / 1e12:.1f} TFLOP/s ({f2 / t2 / 2.5e15 * 100:.1f}% of 2.5 PFLOP/s); "
          f"algorithmic flops {f2:.3e}", flush=True)


    # one token (decode): matrix-vector kernels, bound by the read of the weights.  The weights of 12 "layers" are
    # cycled through (about 1 GB), so that they come from HBM and not from the 256 MB last-level cache.
    x1, q1, k1, v1, y1 = x[:1].contiguous(), q[:, :1].contiguous(), k[:, :1].contiguous(), v[:, :1].contiguous(), y[:1].contiguous()
    ws_, wos_ = [w.clone() for _ in range(12)], [wo.clone() for _ in range(12)]

    def timed_cycle(fn, n=60):
        for i in range(12):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i % 12)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n * 1e-3

    t3 = timed_cycle(lambda i: hb.hi_qkv_rope(s, x1, ws_[i], D, Hq, Hkv, 1, a.past, 500000.0, 0, q1, k1, v1, None))
    t4 = timed_cycle(lambda i: hb.hi_out_proj(s, q1, wos_[i], Hq, D, 1, 0, y1))
    b3, b4 = w.numel() * 2.0, wo.numel() * 2.0
    print(f"qkv+rope  C=1: {t3 * 1e6:.1f} us, {b3 / t3 / 1e9:.0f} GB/s ({b3 / t3 / 8e12 * 100:.1f}% of 8 TB/s); weight bytes {b3:.3e}", flush=True)
    print(f"out_proj  C=1: {t4 * 1e6:.1f} us, {b4 / t4 / 1e9:.0f} GB/s ({b4 / t4 / 8e12 * 100:.1f}% of 8 TB/s); weight bytes {b4:.3e}", flush=True)


if __name__ == "__main__":
    main()
