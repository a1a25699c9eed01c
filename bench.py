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
# HBM-side bytes per launch come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, each scaled by what the same
# counter read for a 1 GiB copy kernel in the same run.  The prefill figure is read from the profile summary that
# holds it, where it is stored next to the hash of the kernel source it was measured on: a changed kernel or another
# shape gives null instead of a stale number.  The resident decode launch reads each K/V byte once (measured).
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "prefill_kernel_deep_unit_resident_pmc.md")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2502_12574_amd", "csrc", f) for f in ("hi_prefill.hip", "hi_prefill_wide.inc")]
DECODE_TRAFFIC_PER_ROW = 512.0


def prefill_kernel_name():
    if EXTRA_FLAGS & hb.HI_FLAG_PREFILL_MFMA32:
        return "prefill_kernel_deep"
    return "prefill_kernel_deep16" if EXTRA_FLAGS & hb.HI_FLAG_PREFILL_8WAVE else "prefill_kernel_wide"


def prefill_traffic_per_launch(S, C):
    """bytes per staging-slice launch of the dominant kernel, or (None, why)"""
    import hashlib
    import re
    try:
        # fingerprint of the code, not of the text: // comments and white space do not count
        code = re.sub(r"//[^\n]*", "", "".join(open(f, encoding="utf-8").read() for f in KERNEL_SOURCES))
        sha = hashlib.sha256(re.sub(r"\s+", " ", code).encode()).hexdigest()[:16]
        for line in open(TRAFFIC_PROFILE):
            m = re.match(r"\s*bench-traffic: context=(\d+) chunk=(\d+) source_sha256=(\w+) bytes_per_launch=(\d+)", line)
            if m and (int(m.group(1)), int(m.group(2))) == (S, C):
                if m.group(3) == sha:
                    return int(m.group(4)), os.path.relpath(TRAFFIC_PROFILE, ROOT)
                return None, "the kernel source changed after the counter run in " + os.path.relpath(TRAFFIC_PROFILE, ROOT)
    except OSError:
        pass
    return None, "no counter run for this shape"


_T0 = time.perf_counter()


EXTRA_FLAGS = 0      # kernel-selection flags of the command line, added to every flag word set below
Q_PRESCALED = True   # the queries carry the softmax scale (hi_problem.q_prescaled), as the Q projection emits them


def set_flags(ss, flags):
    hb.hi_ctx_set_flags(ss.ctx, flags | EXTRA_FLAGS)


def note(msg):
    """progress line of the work itself (stderr; stdout carries the one JSON line)"""
    print(f"bench.py [{time.perf_counter() - _T0:6.1f} s] {msg}", file=sys.stderr, flush=True)


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
    qs = hb.HI_Q_PRESCALE if Q_PRESCALED else 1.0          # the oracle takes the q of Eq. 3: the drawn query / the constant
    q = synth.to_f64(synth.draw_q(seed, 0, 0, 0, S, scale=qs)[pos]) / qs
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
    # the small configuration in full: 4 query heads over one KV head, 2048 tokens, then 16 decode rows
    n1, nd1 = 2048, 16
    Q1 = np.stack([synth.to_f64(synth.draw_q(seed, 0, g, 0, n1 + nd1, scale=qs)) / qs for g in range(4)])
    K1 = synth.to_f64(synth.draw_k(seed, 0, 0, 0, n1 + nd1))
    V1 = synth.to_f64(synth.draw_v(seed, 0, 0, 0, n1 + nd1))
    t0 = time.perf_counter()
    cache = oa.HeadwiseCache(1, 1, D)
    oa.prefill_chunked(cache, Q1[None, :, :n1], K1[None, None, :n1], V1[None, None, :n1], 512)
    t_pre1 = time.perf_counter() - t0
    t0 = time.perf_counter()
    for t in range(nd1):
        oa.decode_step(cache, Q1[None, :, n1 + t], K1[None, None, n1 + t], V1[None, None, n1 + t])
    t_dec1 = time.perf_counter() - t0
    return {"value": S / prefill_s, "unit": "tokens/s per layer (prefill)", "cores": cores, "kind": "oracle",
            "decode_ms_per_token_per_layer": decode_ms,
            "small_config_full": {"what": "4 query heads / 1 KV head, 2048 tokens in 4 chunks of 512, then 16 decode "
                                          "steps, run in full", "prefill_s": t_pre1,
                                  "prefill_tokens_per_s": n1 / t_pre1, "decode_ms_per_token": t_dec1 / nd1 * 1e3},
            "sample": f"{total_rows} query rows of one head at positions in the last chunk of the {S}-token "
                      f"context, {total_t:.1f} s of fp64 numpy; extrapolated linearly in row-key pairs to "
                      f"{HQ} heads x S(S+1)/2 pairs"}


def run_stack(args):
    """The literal multi-layer configuration: L attention blocks in Algorithm 1's order (chunk -> layer -> head), each
    layer's Q/K/V produced chunk by chunk from hidden states by hi_qkv_rope (directly drawn Q/K/V of 32 layers would
    not fit HBM), one pinned host allocation per layer, a one-head HBM budget for all layers.  One timed pass."""
    from paper_2502_12574_amd.attention_block import AttentionBlock
    dev, S, C, nd, d_model = "cuda:0", args.context, args.chunk, args.decode_tokens, HQ * D
    L, ss = max(1, args.layers), None
    while ss is None:
        try:
            ss = Session(L, HKV, G, S + max(nd, 1), C, mode=hb.HI_MODE_OFFLOAD, out_fp32=0, per_layer_cache=True,
                         q_prescaled=Q_PRESCALED,
                         progress=lambda m: print("bench.py: " + m, file=sys.stderr, flush=True))
        except RuntimeError as e:               # the box refuses to pin that much: fewer layers, figures stay per layer
            print(f"bench.py: {L} layers of pinned cache refused ({str(e)[:80]}); trying {L // 2}", file=sys.stderr, flush=True)
            torch.cuda.empty_cache()
            L //= 2
            if L < 1:
                raise
    print(f"bench.py: {L} layers, {ss.plan.host_bytes_total / 2**30:.0f} GiB of pinned cache", file=sys.stderr, flush=True)
    blocks = []
    for l in range(L):
        w_qkv = synth.draw_weight(args.seed, synth.TENSOR_WQKV, l, (HQ + 2 * HKV) * D, d_model, device=dev)
        w_o = synth.draw_weight(args.seed, synth.TENSOR_WO, l, d_model, HQ * D, device=dev)
        blocks.append(AttentionBlock(ss, l, w_qkv, w_o))
    starts = list(range(0, S, C))
    xs = [synth.draw_hidden(args.seed, 0, p, min(C, S - p), d_model, device=dev) for p in starts]
    xbuf = [torch.empty(C, d_model, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    first = blocks[0].calls[0]
    set_flags(ss, hb.HI_FLAG_TIME_KERNELS)
    hb.hi_reset_stats(ss.ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for ci, p in enumerate(starts):
        n = xs[ci].shape[0]
        x = xs[ci]
        for l in range(L):
            if l + 1 < L:
                nxt = (l + 1, first[0], first[1], p)
            elif ci + 1 < len(starts):
                nxt = (0, first[0], first[1], p + n)
            else:
                nxt = (0, first[0], first[1], S) if nd else None
            y = xbuf[l & 1][:n]
            blocks[l].forward(x, p, y, nxt)
            with torch.cuda.stream(ss.s_compute):
                y.add_(x)                      # the residual connection keeps the hidden states at unit scale
            x = y
        if ci % 8 == 7:
            print(f"bench.py: chunk {ci + 1} of {len(starts)} enqueued, {time.perf_counter() - t0:.0f} s", file=sys.stderr, flush=True)
    ss.sync()
    t_pre = time.perf_counter() - t0
    st = ss.stats()
    hb.hi_reset_stats(ss.ctx)
    xd = synth.draw_hidden(args.seed, 0, S, nd + 1, d_model, device=dev)[:, None]
    t0 = time.perf_counter()
    for t in range(nd):
        x = xd[t]
        for l in range(L):
            nxt = (l + 1, first[0], first[1], S + t) if l + 1 < L else ((0, first[0], first[1], S + t + 1) if t + 1 < nd else None)
            y = xbuf[l & 1][:1]
            blocks[l].forward(x, S + t, y, nxt)
            with torch.cuda.stream(ss.s_compute):
                y.add_(x)
            x = y
    ss.sync()
    t_dec = time.perf_counter() - t0
    sd = ss.stats()
    flops = causal_flops_layer(S)
    kern_s = st.prefill_kernel_ms * 1e-3 / L
    dec_ms = t_dec / max(nd, 1) / L * 1e3
    result = {
        "metric": "prefill tokens/s per layer at 1M ctx (decode ms/token per layer and roofline fractions alongside)",
        "value": S / (t_pre / L), "unit": "tokens/s per layer", "n_gpus": 1, "steps": 1, "warmup": 0,
        "ms_per_step": (t_pre + t_dec) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 inputs, fp32 accumulate (MFMA)", "data": "synthetic",
        "config": {"workload": f"{L}-layer attention stack (attention blocks only, no MLP), Llama-3-8B shapes: {HQ} Q / {HKV} KV "
                               f"heads, head_dim {D}, d_model {d_model}, context {S}, chunk {C}, loop chunk -> layer -> head, "
                               f"{nd} decode tokens; each layer's Q/K/V come from hi_qkv_rope on the hidden states, the "
                               f"layer's output from hi_out_proj; {ss.plan.host_bytes_total / 2**30:.0f} GiB of K/V in "
                               f"pinned host DRAM (one allocation per layer), 1-KV-head HBM budget",
                   "context": S, "chunk": C, "decode_tokens": nd, "layers_timed": L, "layers_asked": args.layers,
                   "q_prescaled": Q_PRESCALED, "seed": args.seed},
        "prefill_s_total": t_pre, "prefill_s_per_layer": t_pre / L,
        "decode_ms_per_token_per_layer_offloaded": dec_ms if nd else None,
        "decode_link": {"achieved_GBps": 512.0 * HKV * S / (dec_ms * 1e-3) / 1e9 if nd else None, "peak_GBps": PEAK_LINK_GBPS},
        "peak_staging_bytes": max(st.peak_staging_bytes, sd.peak_staging_bytes), "one_head_bytes": ss.plan.host_bytes_per_head,
        "bytes_h2d_prefill": st.bytes_h2d, "bytes_d2h_prefill": st.bytes_d2h,
        "roofline": {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / kern_s / 1e12 / PEAK_MFMA_TFLOPS, "traffic": None, "kernel": prefill_kernel_name(),
                     "launches_per_step": st.n_prefill_kernels, "avg_launch_ms": st.prefill_kernel_ms / max(st.n_prefill_kernels, 1),
                     "wall_TFLOPs": flops / (t_pre / L) / 1e12,
                     "note": "wall time includes the projections of every chunk and layer (about 1.2 % of a layer)"},
        "overlap": {"t_pipelined_s": t_pre / L, "t_kernel_sum_pipelined_s": kern_s,
                    "h2d_copy_engine_s": st.h2d_copy_ms * 1e-3 / L, "d2h_copy_engine_s": st.d2h_copy_ms * 1e-3 / L,
                    "compute_stream_between_kernels_s": st.exposed_copy_ms * 1e-3 / L,
                    "hidden_fraction_from_stream_idle": 1.0 - st.exposed_copy_ms / max(st.h2d_copy_ms, 1e-9)},
    }
    ss.close()
    print(json.dumps(result))


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
    ap.add_argument("--no-next-legs", action="store_true", help="skip the streaming-heads, projection and 4-bit-link legs")
    ap.add_argument("--layers", type=int, default=1, help="layers run in Algorithm 1's order (chunk -> layer -> head); "
                    "every figure stays per layer")
    ap.add_argument("--heads-per-call", type=int, default=0, help="KV heads per call; 0 = what hi_offload_plan "
                    "recommends for the context (Section 4, adaptive head-wise offloading: 1 beyond 256K tokens)")
    ap.add_argument("--seed", type=int, default=20250216)
    ap.add_argument("--resident-passes", type=int, default=2, help="passes of the compute-only (HBM-resident) prefill leg; "
                    "the last one is timed")
    ap.add_argument("--no-q-prescale", action="store_true", help="hand the attention calls plain queries (the q of Eq. 3) "
                    "instead of queries that carry the softmax scale; one more multiplication per score in the kernels")
    ap.add_argument("--mfma32", action="store_true", help="the 8-wave prefill kernel in its 32x32x16 MFMA form (A/B runs)")
    ap.add_argument("--eight-wave", action="store_true", help="the 16x16x32 prefill kernel with 8 wavefronts of 32 query rows in every launch (A/B runs)")
    ap.add_argument("--single-slices", action="store_true", help="one attention launch per staging slice (A/B runs)")
    ap.add_argument("--wide", action="store_true", help="the 16x16x32 prefill kernel with 4 wavefronts of 64 query rows in every launch (A/B runs)")
    ap.add_argument("--peaked-keys", action="store_true", help="one key row in ten scaled x4 (peaked softmax rows)")
    ap.add_argument("--no-kernel-timing", action="store_true", help="run the timed steps without the library's HIP events "
                    "around kernels and copies (wall figures only; the roofline object is then empty)")
    ap.add_argument("--stack", action="store_true", help="the literal multi-layer configuration: --layers attention blocks "
                    "whose Q/K/V come from the projections of hidden states, one pinned allocation per layer, one pass")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); --gpus must be 1. KV heads are "
              "independent, so N GPUs would each own n_kv_heads/N heads and their own host link.", file=sys.stderr)
        sys.exit(2)
    global EXTRA_FLAGS, Q_PRESCALED
    Q_PRESCALED = not args.no_q_prescale
    EXTRA_FLAGS = (hb.HI_FLAG_PREFILL_MFMA32 if args.mfma32 else 0) | (hb.HI_FLAG_PREFILL_8WAVE if args.eight_wave else 0) | (hb.HI_FLAG_PREFILL_WIDE if args.wide else 0) | (hb.HI_FLAG_PREFILL_SINGLE_SLICES if args.single_slices else 0)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)

    if args.stack:
        return run_stack(args)
    dev = "cuda:0"
    S, C, nd = args.context, args.chunk, args.decode_tokens
    S_max = S + max(nd, args.resident_decode_tokens)
    NL = max(1, args.layers)
    ss = Session(NL, HKV, G, S_max, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=0, q_prescaled=Q_PRESCALED)
    hpc = args.heads_per_call if args.heads_per_call > 0 else max(1, ss.plan.heads_per_group)
    t_gen = time.perf_counter()
    with torch.cuda.stream(ss.s_compute):
        inp = driver.LayerInputs(args.seed, NL, HKV, G, S, C, dev, peaked=args.peaked_keys,
                                 q_scale=hb.HI_Q_PRESCALE if Q_PRESCALED else 1.0)
        dec_rows = [inp.decode_rows(S + t) for t in range(max(nd, args.resident_decode_tokens))]
        out_buf = [torch.empty(HKV, G, C, D, dtype=ss.out_dtype, device=dev) for _ in range(NL)]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    note(f"inputs drawn ({t_gen:.1f} s)")

    # runs of minutes report their progress (the host is never more than two units ahead of the GPU)
    n_chunks = (S + C - 1) // C
    every = max(1, n_chunks // 8)
    progress = (lambda c, l, h, out: note(f"chunk {c + 1} of {n_chunks} enqueued")
                if h == HKV - 1 and l == NL - 1 and c % every == every - 1 else None) if S * NL >= (1 << 21) else None

    def step(timed):
        hb.hi_reset_stats(ss.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.prefill(ss, inp, out_buf=out_buf, last_hint=(0, 0, S) if nd else None, heads_per_call=hpc,
                           keep=progress)
        ss.sync()
        t1 = time.perf_counter()
        st_pre = ss.stats()                    # the prefill's own counters and event timings
        hb.hi_reset_stats(ss.ctx)
        t1b = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.decode(ss, inp, S, nd, rows=dec_rows, heads_per_call=hpc)
        ss.sync()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        note(f"step done: prefill {t1 - t0:.3f} s, {nd} decode tokens {t2 - t1b:.3f} s")
        return t1 - t0, t2 - t1b, st_pre, ss.stats()

    set_flags(ss, 0 if args.no_kernel_timing else hb.HI_FLAG_TIME_KERNELS)
    for _ in range(args.warmup):
        step(False)
    pre_s, dec_s, kern_pre_ms, kern_dec_ms, n_pre_k, n_dec_k = [], [], 0.0, 0.0, 0, 0
    copy_ms = {"h2d": 0.0, "d2h": 0.0, "exposed": 0.0}
    bytes_h2d = 0
    peak_staging = 0
    torch.cuda.synchronize()
    t_all0 = time.perf_counter()
    for _ in range(args.steps):
        a, b, st, st_dec = step(True)
        pre_s.append(a); dec_s.append(b)
        kern_pre_ms += st.prefill_kernel_ms; kern_dec_ms += st_dec.decode_kernel_ms
        n_pre_k += st.n_prefill_kernels; n_dec_k += st_dec.n_decode_kernels
        bytes_h2d = st.bytes_h2d
        copy_ms["h2d"] += st.h2d_copy_ms; copy_ms["d2h"] += st.d2h_copy_ms; copy_ms["exposed"] += st.exposed_copy_ms
        peak_staging = max(peak_staging, st.peak_staging_bytes, st_dec.peak_staging_bytes)
    torch.cuda.synchronize()
    t_all = time.perf_counter() - t_all0
    K = max(args.steps, 1)
    prefill_s = sum(pre_s) / K / NL                       # per layer
    decode_ms_tok = (sum(dec_s) / K) / max(nd, 1) * 1e3 / NL
    flops = causal_flops_layer(S)
    kern_s = max(kern_pre_ms, 1e-9) / K * 1e-3 / NL

    extra = {}
    if not args.no_extra_legs:
        # transfer-only: the same copy sequence with the kernels disabled
        set_flags(ss, hb.HI_FLAG_SKIP_KERNELS)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(ss.s_compute):
            driver.prefill(ss, inp, out_buf=out_buf, heads_per_call=hpc)
        ss.sync()
        t_xfer = (time.perf_counter() - t0) / NL
        note(f"transfer-only leg done ({t_xfer:.3f} s per layer)")
        set_flags(ss, hb.HI_FLAG_TIME_KERNELS)
        link_bytes = 512.0 * HKV * sum(range(0, S, C)) + 512.0 * HKV * S
        # compute-only: the same calls on one layer with K/V resident in HBM (no link, no ring; a unit's past is one
        # contiguous segment there, so it takes one launch instead of one per staging slice)
        ss_r = Session(1, HKV, G, S_max, C, mode=hb.HI_MODE_RESIDENT, out_fp32=0, q_prescaled=Q_PRESCALED)
        inp0 = inp.single_layer(0)

        def resident_prefill():
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with torch.cuda.stream(ss_r.s_compute):
                driver.prefill(ss_r, inp0, out_buf=out_buf[:1], heads_per_call=hpc, keep=progress if NL == 1 else None)
            ss_r.sync()
            return time.perf_counter() - t0

        # (the first pass also fills the resident cache for the decode leg below; with --resident-passes 1 it is the
        # timed one - the kernels are warm from the steps above)
        for _ in range(max(1, args.resident_passes)):
            t_comp = resident_prefill()
            note(f"compute-only pass done ({t_comp:.3f} s)")
        # hidden = 1 - max(0, T_pipelined - T_compute_only) / T_transfer_only; two more readings of the same thing ride
        # along: with the summed kernel time of the pipelined run in place of the resident run, and the time the
        # compute stream spent between attention launches (launch latency included) over the transfer time
        exposed_s = copy_ms["exposed"] / K * 1e-3 / NL
        extra["overlap"] = {"t_pipelined_s": prefill_s, "t_compute_only_s": t_comp, "t_transfer_only_s": t_xfer,
                            "hidden_fraction": 1.0 - max(0.0, prefill_s - t_comp) / t_xfer,
                            "compute_only": "the same calls on one layer with K/V resident in HBM, wall time",
                            "t_kernel_sum_pipelined_s": kern_s,
                            "hidden_fraction_vs_kernel_sum": 1.0 - max(0.0, prefill_s - kern_s) / t_xfer,
                            "compute_stream_between_kernels_s": exposed_s,
                            "hidden_fraction_from_stream_idle": 1.0 - exposed_s / t_xfer,
                            "h2d_copy_engine_s": copy_ms["h2d"] / K * 1e-3 / NL,
                            "d2h_copy_engine_s": copy_ms["d2h"] / K * 1e-3 / NL,
                            "link_bytes": link_bytes, "transfer_only_GBps": link_bytes / t_xfer / 1e9}
        # HBM-resident decode over the cache the resident prefill has just filled
        set_flags(ss_r, hb.HI_FLAG_TIME_KERNELS)
        nr = args.resident_decode_tokens
        # all KV heads of the layer in one call per token (head groups; with everything in HBM nothing speaks
        # against the largest group)
        grp = [(r[0][0], r[1][0], r[2][0]) for r in dec_rows[:nr]]          # layer 0, heads stacked
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
        note("resident decode leg done")

    traffic, traffic_src = prefill_traffic_per_launch(S, C)
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
                               f"budget" + ("; queries carry the softmax scale, as the Q projection emits them" if Q_PRESCALED else ""),
                   "context": S, "chunk": C, "decode_tokens": nd, "layers_timed": NL, "heads_per_call": hpc,
                   "peaked_keys": bool(args.peaked_keys), "q_prescaled": Q_PRESCALED,
                   "seed": args.seed},
        "prefill_s_per_layer": prefill_s,
        "decode_ms_per_token_per_layer_offloaded": decode_ms_tok if nd else None,
        "decode_link": {"achieved_GBps": dec_link_GBps, "peak_GBps": PEAK_LINK_GBPS,
                        "frac": dec_link_GBps / PEAK_LINK_GBPS if nd else None},
        "peak_staging_bytes": peak_staging, "one_head_bytes": ss.plan.host_bytes_per_head,
        "input_generation_s": t_gen,
        "roofline": {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / kern_s / 1e12 / PEAK_MFMA_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": prefill_kernel_name(),
                     "launches_per_step": n_pre_k / K, "avg_launch_ms": kern_pre_ms / max(n_pre_k, 1),
                     "flops_per_launch": flops * NL / (n_pre_k / K),
                     "wall_TFLOPs": flops / prefill_s / 1e12},
    }
    result.update(extra)
    ss.close()
    del ss
    if not args.no_extra_legs and not args.no_next_legs:
        # the rows built after the hot path met its bar: streaming heads (Appendix E: 4 of the 8 heads keep sink +
        # recent tokens in HBM) on the same layer, and the projections either side of the attention calls
        from paper_2502_12574_amd import layer_bench, proj_bench
        torch.cuda.empty_cache()
        sp = layer_bench.run(S, C, HKV // 2, 128, 512, 8, HKV // 2, heads_per_call=hpc, q_prescaled=Q_PRESCALED)
        sp["prefill_speedup_vs_all_retrieval"] = prefill_s / sp["prefill_s"]
        if nd:
            sp["decode_speedup_vs_all_retrieval"] = decode_ms_tok / sp["decode_ms_per_token"]
        result["streaming_heads_50pct"] = sp
        note("streaming-heads leg done")
        result["projections"] = proj_bench.measure(C)
        # the same layer with 4-bit rows on the host link (every head offloaded): the link-bound decode should follow
        # the bytes per row, the prefill should not change
        torch.cuda.empty_cache()
        lk = layer_bench.run(S, C, 0, 0, 0, 8, 1, link_kv_bits=4, heads_per_call=hpc, q_prescaled=Q_PRESCALED)
        lk["prefill_speedup_vs_bf16_rows"] = prefill_s / lk["prefill_s"]
        if nd:
            lk["decode_speedup_vs_bf16_rows"] = decode_ms_tok / lk["decode_ms_per_token"]
        result["link_kv_4bit"] = lk
        note("4-bit link leg done")
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.seed, S, C)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
