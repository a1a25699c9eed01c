"""Projection micro-benchmark: the Q/K/V projection with rotary embedding (hi_qkv_rope) and the output projection
(hi_out_proj) of one chunk at Llama-3-8B shapes (d_model 4096, 32 query / 8 KV heads), HIP-event timed.

    python -m paper_2502_12574_amd.proj_bench [--chunk 16384] [--reps 10] [--past 1032192]

Algorithmic flops: 2 * chunk * d_model * (Hq + 2 Hkv) * 128 and 2 * chunk * (Hq * 128) * d_model.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as hb


def measure(C=16384, D=4096, Hq=32, Hkv=8, past=(1 << 20) - 16384, reps=10, dev="cuda:0"):
    """Time both projections for a chunk of C tokens and for one token; returns a dict of seconds, rates, fractions."""
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

    def timed(fn, n, cycle=1):
        for i in range(cycle):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i % cycle)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n * 1e-3

    t1 = timed(lambda i: hb.hi_qkv_rope(s, x, w, D, Hq, Hkv, C, past, 500000.0, 0, q, k, v, ws), reps)
    t2 = timed(lambda i: hb.hi_out_proj(s, q, wo, Hq, D, C, 0, y), reps)
    f1, f2 = 2.0 * C * D * (Hq + 2 * Hkv) * 128, 2.0 * C * Hq * 128 * D
    # one token (decode): matrix-vector kernels, bound by the read of the weights.  The weights of 12 "layers" are
    # cycled through (about 1 GB), so that they come from HBM and not from the 256 MB last-level cache.
    x1, q1, k1, v1, y1 = x[:1].contiguous(), q[:, :1].contiguous(), k[:, :1].contiguous(), v[:, :1].contiguous(), y[:1].contiguous()
    ws_, wos_ = [w.clone() for _ in range(12)], [wo.clone() for _ in range(12)]
    t3 = timed(lambda i: hb.hi_qkv_rope(s, x1, ws_[i], D, Hq, Hkv, 1, past, 500000.0, 0, q1, k1, v1, None), 60, 12)
    t4 = timed(lambda i: hb.hi_out_proj(s, q1, wos_[i], Hq, D, 1, 0, y1), 60, 12)
    b3, b4 = w.numel() * 2.0, wo.numel() * 2.0
    return {"chunk": C, "d_model": D, "q_heads": Hq, "kv_heads": Hkv,
            "qkv_rope": {"s": t1, "flops": f1, "TFLOPs": f1 / t1 / 1e12, "frac_of_mfma_peak": f1 / t1 / 2.5e15},
            "out_proj": {"s": t2, "flops": f2, "TFLOPs": f2 / t2 / 1e12, "frac_of_mfma_peak": f2 / t2 / 2.5e15},
            "qkv_rope_one_token": {"s": t3, "weight_bytes": b3, "GBps": b3 / t3 / 1e9, "frac_of_hbm_peak": b3 / t3 / 8e12},
            "out_proj_one_token": {"s": t4, "weight_bytes": b4, "GBps": b4 / t4 / 1e9, "frac_of_hbm_peak": b4 / t4 / 8e12}}


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
    r = measure(a.chunk, a.d_model, a.q_heads, a.kv_heads, a.past, a.reps)
    for name in ("qkv_rope", "out_proj"):
        m = r[name]
        print(f"{name:9s} C={a.chunk}: {m['s'] * 1e3:.3f} ms, {m['TFLOPs']:.1f} TFLOP/s ({m['frac_of_mfma_peak'] * 100:.1f}% of "
              f"2.5 PFLOP/s); algorithmic flops {m['flops']:.3e}", flush=True)
    for name in ("qkv_rope_one_token", "out_proj_one_token"):
        m = r[name]
        print(f"{name:9s}: {m['s'] * 1e6:.1f} us, {m['GBps']:.0f} GB/s ({m['frac_of_hbm_peak'] * 100:.1f}% of 8 TB/s); "
              f"weight bytes {m['weight_bytes']:.3e}", flush=True)


if __name__ == "__main__":
    main()
