#!/usr/bin/env python3
"""Benchmark of the head-wise offloaded attention path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input: the head-wise chunked prefill of
ONE Llama-3-8B-shaped attention layer (32 query heads / 8 KV heads, head_dim 128) at a 1M-token context (chunk
16384, K/V offloaded per head to pinned host DRAM, at most one KV head of K/V in HBM), followed by decode steps
over the 1M-token offloaded cache.  The layers of an attention-only stack are independent, so the per-layer
figures of the 32-layer configuration are those of one layer.

Prints ONE JSON line.  `value` is prefill tokens/s per layer; decode ms/token per layer (offloaded and
HBM-resident), the MFMA / HBM / host-link roofline fractions and the CPU-oracle baseline ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2502_12574_amd import binding as hb  # noqa: E402
from paper_2502_12574_amd import driver, synth  # noqa: E402
from paper_2502_12574_amd.session import Session  # noqa: E402

HQ, HKV, G, D = 32, 8, 4, 128
PEAK_MFMA_TFLOPS = 2500.0     # dense bf16
PEAK_HBM_GBPS = 8000.0
PEAK_LINK_GBPS = 64.0         # PCIe Gen5 x16, one direction
# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/*_pmc.md), each scaled by
# what the same counter read for a 1 GiB copy kernel in the same run: a prefill launch over one 262144-row
# staging slice with chunk 16384, and the resident decode launch over 1M rows (reads each K/V byte once).
PREFILL_TRAFFIC_PER_LAUNCH = 1103.8 * 2 ** 20 + 16 * 2 ** 20
DECODE_TRAFFIC_PER_ROW = 512.0


def causal_flops_layer(S):
    return 4.0 * D * HQ * (S * (S + 1) / 2.0)


def cpu_baseline(seed, S, C, seconds_target=15.0):
    """The fp64 oracle, as it stands, on a bounded sample: query rows of one query head spread over the last chunk
    of the context (so nearly every computed row-key pair is a causal one), extrapolated linearly in row-key pairs
    to one layer's prefill."""
    from oracle import attention as oa
    cores = len(os.sched_getaffinity(0))
    torch.set_num_threads(cores)
    K = synth.to_f64(synth.draw_k(seed, 0, 0, 0, S))
    V = synth.to_f64(synth.draw_v(seed, 0, 0, 0, S))
    rows = 64
    pos = np.linspace(S - C, S - 1, rows).astype(np.int64)
    q = synth.to_f64(synth.draw_q(seed, 0, 0, 0, S)[pos])
    t0 = time.perf_counter()
    oa.attn_rows(q, K, V, pos)
    dt = time.perf_counter() - t0
    reps, total_rows, total_t = 1, rows, dt
    while total_t < seconds_target and reps < 64:
        t0 = time.perf_counter()
        oa.attn_rows(q, K, V, pos)
        total_t += time.perf_counter() - t0
        total_rows += rows
        reps += 1
    pairs = float(total_rows) * S                       # the oracle scores every key up to the largest position
    sec_per_pair = total_t / pairs
    layer_pairs = HQ * (S * (S + 1) / 2.0)
    prefill_s = sec_per_pair * layer_pairs
    decode_ms = sec_per_pair * HQ * S * 1e3
    return {"value": S / prefill_s, "unit": "tokens/s per layer (prefill)", "cores": cores, "kind": "oracle",
            "decode_ms_per_token_per_layer": decode_ms,
            "sample": f"{total_rows} query rows of one head at positions in the last chunk of the {S}-token "
                      f"context, {total_t:.1f} s of fp64 numpy; extrapolated linearly in row-key pairs to "
                      f"{HQ} heads x S(S+1)/2 pairs"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--context", type=int, default=1 << 20)
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--decode-tokens", type=int, default=16)
    ap.add_argument("--resident-decode-tokens", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true", help="skip transfer-only and resident-decode legs")
    ap.add_argument("--layers", type=int, default=1, help="layers run in Algorithm 1's order (chunk -> layer -> head); "
                    "every figure stays per layer")
    ap.add_argument("--seed", type=int, default=20250216)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); --gpus must be 1. KV heads are "
              "independent, so N GPUs would each own n_kv_heads/N heads and their own host link.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)

    dev = "cuda:0"
    S, C, nd = args.context, args.chunk, args.decode_tokens
    S_max = S + max(nd, args.resident_decode_tokens)
    NL = max(1, args.layers)
    ss = Session(NL, HKV, G, S_max, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=0)
    t_gen = time.perf_counter()
    with torch.cuda.stream(ss.s_compute):
        inp = driver.LayerInputs(args.seed, NL, HKV, G, S, C, dev)
        dec_rows = [inp.decode_rows(S + t) for t in range(max(nd, args.resident_decode_tokens))]
        out_buf = [[torch.empty(G, C, D, dtype=ss.out_dtype, device=dev) for _ in range(HKV)] for _ in range(NL)]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    def step(timed):
        hb.hi_reset_stats(ss.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.prefill(ss, inp, out_buf=out_buf, last_hint=(0, 0, S) if nd else None)
        ss.sync()
        t1 = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.decode(ss, inp, S, nd, rows=dec_rows)
        ss.sync()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1, ss.stats()

    hb.hi_ctx_set_flags(ss.ctx, hb.HI_FLAG_TIME_KERNELS)
    for _ in range(args.warmup):
        step(False)
    pre_s, dec_s, kern_pre_ms, kern_dec_ms, n_pre_k, n_dec_k = [], [], 0.0, 0.0, 0, 0
    bytes_h2d = 0
    peak_staging = 0
    torch.cuda.synchronize()
    t_all0 = time.perf_counter()
    for _ in range(args.steps):
        a, b, st = step(True)
        pre_s.append(a); dec_s.append(b)
        kern_pre_ms += st.prefill_kernel_ms; kern_dec_ms += st.decode_kernel_ms
        n_pre_k += st.n_prefill_kernels; n_dec_k += st.n_decode_kernels
        bytes_h2d = st.bytes_h2d
        peak_staging = max(peak_staging, st.peak_staging_bytes)
    torch.cuda.synchronize()
    t_all = time.perf_counter() - t_all0
    K = max(args.steps, 1)
    prefill_s = sum(pre_s) / K / NL                       # per layer
    decode_ms_tok = (sum(dec_s) / K) / max(nd, 1) * 1e3 / NL
    flops = causal_flops_layer(S)
    kern_s = kern_pre_ms / K * 1e-3 / NL

    extra = {}
    if not args.no_extra_legs:
        # transfer-only: the same copy sequence with the kernels disabled
        hb.hi_ctx_set_flags(ss.ctx, hb.HI_FLAG_SKIP_KERNELS)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.prefill(ss, inp, out_buf=out_buf)
        ss.sync()
        t_xfer = (time.perf_counter() - t0) / NL
        stx = ss.stats()
        hb.hi_ctx_set_flags(ss.ctx, hb.HI_FLAG_TIME_KERNELS)
        link_bytes = 512.0 * HKV * sum(range(0, S, C)) + 512.0 * HKV * S
        hidden = 1.0 - max(0.0, prefill_s - kern_s) / t_xfer
        extra["overlap"] = {"t_pipelined_s": prefill_s, "t_compute_only_s": kern_s, "t_transfer_only_s": t_xfer,
                            "hidden_fraction": hidden, "link_bytes": link_bytes,
                            "transfer_only_GBps": link_bytes / t_xfer / 1e9}
        # HBM-resident decode over the same cache (device copy of the host cache)
        ss_r = Session(1, HKV, G, S_max, C, mode=hb.HI_MODE_RESIDENT, out_fp32=0)
        ss_r.kv.copy_(ss.kv[:ss_r.kv.numel()], non_blocking=False)        # layer 0
        hb.hi_ctx_set_flags(ss_r.ctx, hb.HI_FLAG_TIME_KERNELS)
        nr = args.resident_decode_tokens
        # all KV heads of the layer in one call per token (head groups; with everything in HBM nothing speaks
        # against the largest group)
        grp = [(torch.stack([r[0][0][h] for h in range(HKV)]), torch.stack([r[1][0][h] for h in range(HKV)]),
                torch.stack([r[2][0][h] for h in range(HKV)])) for r in dec_rows[:nr]]
        out_r = torch.empty(HKV, G, D, dtype=ss_r.out_dtype, device=dev)

        def resident_decode(n):
            with torch.cuda.stream(ss_r.s_compute):
                for t in range(n):
                    ss_r.decode_group(0, 0, HKV, grp[t][0], grp[t][1], grp[t][2], S + t, out_r)
            ss_r.sync()

        resident_decode(min(4, nr))
        hb.hi_reset_stats(ss_r.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        resident_decode(nr)
        t_res = time.perf_counter() - t0
        st_r = ss_r.stats()
        k2_ms = st_r.decode_kernel_ms / max(st_r.n_decode_kernels, 1)
        k2_bytes = 512.0 * HKV * (S + (nr - 1) / 2.0)            # one launch covers the 8 heads
        extra["decode_resident"] = {
            "ms_per_token_per_layer": t_res / nr * 1e3,
            "roofline": {"bound": "hbm", "achieved": k2_bytes / (k2_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS,
                         "unit": "GB/s", "frac": k2_bytes / (k2_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                         "traffic": DECODE_TRAFFIC_PER_ROW * HKV * (S + (nr - 1) / 2.0),
                         "kernel": "decode_partial_kernel", "heads_per_launch": HKV, "avg_launch_ms": k2_ms,
                         "wall_GBps": 512.0 * HKV * S * nr / t_res / 1e9}}
        ss_r.close()
        del ss_r

    dec_link_GBps = 512.0 * HKV * (S + (nd - 1) / 2.0) / (decode_ms_tok * 1e-3) / 1e9 if nd else None
    result = {
        "metric": "prefill tokens/s per layer at 1M ctx (decode ms/token per layer and roofline fractions alongside)",
        "value": S / prefill_s,
        "unit": "tokens/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_all / K * 1e3,                    # one step = prefill + decode tokens of all timed layers
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 inputs, fp32 accumulate (MFMA)", "data": "synthetic",
        "config": {"workload": f"one Llama-3-8B-shaped attention layer of the 32-layer 1M-token configuration: "
                               f"{HQ} Q / {HKV} KV heads, head_dim {D}, context {S}, head-wise chunked prefill "
                               f"chunk {C} + {nd} decode tokens, K/V offloaded to pinned host DRAM, 1-KV-head HBM "
                               f"budget", "context": S, "chunk": C, "decode_tokens": nd, "layers_timed": NL,
                   "seed": args.seed},
        "prefill_s_per_layer": prefill_s,
        "decode_ms_per_token_per_layer_offloaded": decode_ms_tok if nd else None,
        "decode_link": {"achieved_GBps": dec_link_GBps, "peak_GBps": PEAK_LINK_GBPS,
                        "frac": dec_link_GBps / PEAK_LINK_GBPS if nd else None},
        "peak_staging_bytes": peak_staging, "one_head_bytes": ss.plan.host_bytes_per_head,
        "input_generation_s": t_gen,
        "roofline": {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / kern_s / 1e12 / PEAK_MFMA_TFLOPS,
                     "traffic": PREFILL_TRAFFIC_PER_LAUNCH if (S, C) == (1 << 20, 16384) else None,
                     "kernel": "prefill_kernel_deep",
                     "launches_per_step": n_pre_k / K, "avg_launch_ms": kern_pre_ms / max(n_pre_k, 1),
                     "flops_per_launch": flops * NL / (n_pre_k / K),
                     "wall_TFLOPs": flops / prefill_s / 1e12},
    }
    result.update(extra)
    ss.close()
    del ss
    if not args.no_extra_legs:
        # the rows built after the hot path met its bar: streaming heads (Appendix E: 4 of the 8 heads keep sink +
        # recent tokens in HBM) on the same layer, and the projections either side of the attention calls
        from paper_2502_12574_amd import layer_bench, proj_bench
        torch.cuda.empty_cache()
        sp = layer_bench.run(S, C, HKV // 2, 128, 512, 8, HKV // 2)
        sp["prefill_speedup_vs_all_retrieval"] = prefill_s / sp["prefill_s"]
        if nd:
            sp["decode_speedup_vs_all_retrieval"] = decode_ms_tok / sp["decode_ms_per_token"]
        result["streaming_heads_50pct"] = sp
        result["projections"] = proj_bench.measure(C)
        # the same layer with 4-bit rows on the host link (every head offloaded): the link-bound decode should follow
        # the bytes per row, the prefill should not change
        torch.cuda.empty_cache()
        lk = layer_bench.run(S, C, 0, 0, 0, 8, 1, link_kv_bits=4)
        lk["prefill_speedup_vs_bf16_rows"] = prefill_s / lk["prefill_s"]
        if nd:
            lk["decode_speedup_vs_bf16_rows"] = decode_ms_tok / lk["decode_ms_per_token"]
        result["link_kv_4bit"] = lk
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.seed, S, C)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
