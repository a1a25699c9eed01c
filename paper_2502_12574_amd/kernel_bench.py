#!/usr/bin/env python3
"""Kernel-level micro-benchmark: one HBM-resident prefill unit and one decode unit, HIP-event timed.

    python3 paper_2502_12574_amd/kernel_bench.py [--past P] [--chunk C] [--reps R] [--what prefill|decode|both|kvq]
                                                 [--narrow|--deep] [--calibrate] [--rows N] [--gqa G]

Used for the rocprofv3 counter runs under profiles/ (--calibrate adds a plain 1 GiB device copy whose FETCH_SIZE /
WRITE_SIZE readings give the scale of those counters).  K/V are resident in HBM, so this isolates K1 / K2+K3 from
the host link.  --what kvq times the two conversions of the 4-bit link rows alone (hi_kv_quantize / hi_kv_dequantize
over --rows rows, cycling through buffers larger than the last-level cache) next to a plain device copy.
"""
from __future__ import annotations

import argparse
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from paper_2502_12574_amd import binding as hb  # noqa: E402
from paper_2502_12574_amd import synth  # noqa: E402
from paper_2502_12574_amd.session import Session  # noqa: E402


def kvq(n, reps, calibrate, dev):
    s = torch.cuda.current_stream()
    if calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        dst.copy_(src)
        print("calibration: one device copy kernel reading 1 GiB and writing 1 GiB", flush=True)
        del src, dst
    n_buf = max(2, (768 << 20) // (n * 336) + 1)
    rows = [torch.randn(n, 128, device=dev).to(torch.bfloat16) for _ in range(n_buf)]
    packed = [torch.empty(n, 80, dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, what, nbytes):
        fn(0)
        e0.record()
        for _ in range(reps):
            for i in range(n_buf):
                fn(i)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * n_buf)
        print(f"{what} of {n} rows: {us:.1f} us/launch, {nbytes / us / 1e6:.2f} TB/s "
              f"({nbytes / us / 1e6 / 8 * 100:.0f}% of 8 TB/s)", flush=True)

    timed(lambda i: hb.hi_kv_quantize(s, rows[i], n, packed[i]), "kv_quant_kernel (256 B in, 80 B out per row)", n * 336)
    timed(lambda i: hb.hi_kv_dequantize(s, packed[i], n, rows[i]), "kv_dequant_kernel (80 B in, 256 B out per row)", n * 336)
    timed(lambda i: rows[i].copy_(rows[(i + 1) % n_buf]), "device copy (256 B in, 256 B out per row)", n * 512)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--past", type=int, default=1 << 20)
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--what", default="both", choices=["prefill", "decode", "both", "kvq"])
    ap.add_argument("--rows", type=int, default=524288, help="rows per conversion launch (--what kvq)")
    ap.add_argument("--gqa", type=int, default=4, choices=[1, 2, 4, 8], help="query heads per KV head")
    ap.add_argument("--narrow", action="store_true", help="force the 4-wave, 2-stage prefill kernel")
    ap.add_argument("--deep", action="store_true", help="force the 8-wave, 4-stage prefill kernel")
    ap.add_argument("--mfma32", action="store_true", help="the 8-wave kernel in its 32x32x16 MFMA form")
    ap.add_argument("--eight-wave", action="store_true", help="the 16x16x32 kernel with 8 wavefronts of 32 query rows")
    ap.add_argument("--wide", action="store_true", help="the 16x16x32 kernel with 4 wavefronts of 64 query rows")
    ap.add_argument("--q-prescaled", action="store_true",
                    help="queries that carry the softmax scale (hi_problem.q_prescaled): no multiplication per score")
    ap.add_argument("--zeros", action="store_true",
                    help="all-zero Q, K, V: the same instruction stream with no switching in the multipliers, i.e. the "
                         "kernel's schedule without the board's power limit")
    ap.add_argument("--calibrate", action="store_true", help="also run a plain 1 GiB device-to-device copy")
    args = ap.parse_args()
    P, C, G, dev = args.past, args.chunk, args.gqa, "cuda:0"
    if args.what == "kvq":
        return kvq(args.rows, args.reps, args.calibrate, dev)
    ss = Session(1, 1, G, P + C, C, mode=hb.HI_MODE_RESIDENT, out_fp32=0, q_prescaled=args.q_prescaled)
    qs = hb.HI_Q_PRESCALE if args.q_prescaled else 1.0
    flags = hb.HI_FLAG_TIME_KERNELS
    flags |= (hb.HI_FLAG_PREFILL_NARROW if args.narrow else 0) | (hb.HI_FLAG_PREFILL_DEEP if args.deep else 0)
    flags |= hb.HI_FLAG_PREFILL_MFMA32 if args.mfma32 else 0
    flags |= hb.HI_FLAG_PREFILL_8WAVE if args.eight_wave else 0
    flags |= hb.HI_FLAG_PREFILL_WIDE if args.wide else 0
    hb.hi_ctx_set_flags(ss.ctx, flags)
    with torch.cuda.stream(ss.s_compute):
        cv = ss.cache_view()
        step = 1 << 18
        for a in range(0, P, step):
            b = min(P, a + step)
            cv[0, 0, 0, a:b] = synth.draw_k(1, 0, 0, a, b - a, device=dev)
            cv[0, 0, 1, a:b] = synth.draw_v(1, 0, 0, a, b - a, device=dev)
        Q = torch.stack([synth.draw_q(1, 0, g, P, C, device=dev, scale=qs) for g in range(G)])
        K = synth.draw_k(1, 0, 0, P, C, device=dev)
        V = synth.draw_v(1, 0, 0, P, C, device=dev)
        if args.zeros:
            cv.zero_(); Q.zero_(); K.zero_(); V.zero_()
        out = torch.empty(G, C, 128, dtype=torch.bfloat16, device=dev)
        outd = torch.empty(G, 128, dtype=torch.bfloat16, device=dev)
        if args.calibrate:
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
            dst = torch.empty_like(src)
            dst.copy_(src)
            print("calibration: one device copy kernel reading 1 GiB and writing 1 GiB", flush=True)
        if args.what in ("prefill", "both"):
            ss.prefill_head(0, 0, Q, K, V, P, out)
            ss.sync()
            hb.hi_reset_stats(ss.ctx)
            for _ in range(args.reps):
                ss.prefill_head(0, 0, Q, K, V, P, out)
            st = ss.stats()
            ms = st.prefill_kernel_ms / st.n_prefill_kernels
            fl = 4.0 * 128 * G * (C * P + C * (C + 1) / 2)
            print(f"prefill unit P={P} C={C} G={G}: {ms:.3f} ms/launch, {fl / ms / 1e9:.1f} TFLOP/s "
                  f"({fl / ms / 1e9 / 2500 * 100:.1f}% of 2.5 PFLOP/s); algorithmic flops/launch {fl:.4g}", flush=True)
        if args.what in ("decode", "both"):
            n = P + C - 1
            q0 = Q[:, 0].contiguous()
            for _ in range(3):
                ss.decode_head(0, 0, q0, K[0], V[0], n, outd)
            ss.sync()
            hb.hi_reset_stats(ss.ctx)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps * 4):
                ss.decode_head(0, 0, q0, K[0], V[0], n, outd)
            e1.record()
            e1.synchronize()
            st = ss.stats()
            ms = st.decode_kernel_ms / st.n_decode_kernels
            print(f"decode unit rows={n}: split-KV kernel {ms * 1e3:.1f} us/launch, {512.0 * n / ms / 1e6:.1f} GB/s "
                  f"({512.0 * n / ms / 1e6 / 8000 * 100:.1f}% of 8 TB/s); algorithmic bytes/launch {512 * n}; "
                  f"whole call {e0.elapsed_time(e1) / (args.reps * 4) * 1e3:.1f} us", flush=True)
    ss.close()


if __name__ == "__main__":
    main()
