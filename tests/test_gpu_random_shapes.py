"""Seeded random sweep over shapes the hand-picked cases may miss: group size, chunk lengths, context, head kinds
(offloaded / resident / streaming), sink and window lengths, modes.  Every output against the fp64 oracles."""
import os
import random

import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import streaming as os_
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import synth
from paper_2502_12574_amd.session import Session

pytestmark = pytest.mark.gpu
MAX_ABS, REL_L2 = 1e-2, 5e-3


def check(got, ref, what):
    got = got.detach().to("cpu").to(torch.float64).numpy()
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    err = float(np.abs(got - ref).max())
    rel = float(np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()))
    assert err <= MAX_ABS and rel <= REL_L2, (what, err, rel)


def draw_case(rng):
    G = rng.choice([1, 2, 4, 4, 4, 8])
    H = rng.choice([2, 3, 4])
    T = rng.choice([0, 0, 1, H - 1])
    n_ret = H - T
    mode = rng.choice([hb.HI_MODE_OFFLOAD, hb.HI_MODE_OFFLOAD, hb.HI_MODE_RESIDENT])
    R = rng.choice([0, 0, 1]) if mode == hb.HI_MODE_OFFLOAD else 0
    R = min(R, n_ret)
    C = rng.choice([37, 64, 100, 128, 200, 256, 333])
    S = rng.randint(1, 900)
    nd = rng.choice([0, 1, 3])
    n_sink = rng.choice([0, 1, 5, 64, 130])
    n_recent = rng.choice([1, 2, 33, 64, 100, 257, 5000])
    group = rng.choice([1, 1, 2])
    # which prefill kernel: the launcher's choice, or one of the forced forms (these shapes are far below the sizes
    # at which the launcher picks the 8-wave kernels by itself)
    flags = rng.choice([0, 0, hb.HI_FLAG_PREFILL_DEEP, hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_PAIRED,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_UNPAIRED,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_8WAVE,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_WIDE, hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_WIDE,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_PAIRED | hb.HI_FLAG_PREFILL_WIDE,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_MFMA32,
                        hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_PAIRED | hb.HI_FLAG_PREFILL_MFMA32,
                        hb.HI_FLAG_PREFILL_NARROW])
    pre = rng.choice([False, False, True])       # queries that carry the softmax scale (hi_problem.q_prescaled)
    return dict(G=G, H=H, T=T, R=R, mode=mode, C=C, S=S, nd=nd, n_sink=n_sink, n_recent=n_recent, group=group,
                flags=flags, pre=pre)


@pytest.mark.parametrize("case_id", range(int(os.environ.get("HI_TEST_RANDOM_CASES", "24"))))
def test_random_shape(case_id):
    rng = random.Random(77000 + case_id)
    c = draw_case(rng)
    G, H, T, R, C, S, nd = c["G"], c["H"], c["T"], c["R"], c["C"], c["S"], c["nd"]
    n_sink, n_recent, dev, seed = c["n_sink"], c["n_recent"], "cuda:0", 77000 + case_id
    n_tok = S + nd
    n_ret = H - T
    max_ctx = max(n_tok, 1024)                     # room for a ring of four 256-row slices
    # calls of a layer: groups inside each kind of head (resident pairs come first among the retrieval heads)
    kinds = [("res" if h < R else "off") for h in range(n_ret)] + ["str"] * T
    calls, h = [], 0
    while h < H:
        nh = 1
        while nh < c["group"] and h + nh < H and kinds[h + nh] == kinds[h]:
            nh += 1
        calls.append((h, nh))
        h += nh
    with Session(1, H, G, max_ctx, C, mode=c["mode"], out_fp32=1, gpu_kv_budget_heads=R + 1, resident_heads=R,
                 streaming_heads=T, sink_tokens=n_sink if T else 0, recent_tokens=n_recent if T else 0,
                 q_prescaled=c["pre"]) as ss:
        hb.hi_ctx_set_flags(ss.ctx, c["flags"])
        ss.kv.view(torch.int16).fill_(0x7FC1)
        if ss.staging is not None:
            ss.staging.view(torch.int16).fill_(0x7FC1)
        pre = {h: [] for h in range(H)}
        dec = {h: [] for h in range(H)}
        with torch.cuda.stream(ss.s_compute):
            qs = hb.HI_Q_PRESCALE if c["pre"] else 1.0
            Q = {h: torch.stack([synth.draw_q(seed, 0, h * G + g, 0, n_tok, device=dev, scale=qs) for g in range(G)])
                 for h in range(H)}
            K = {h: synth.draw_k(seed, 0, h, 0, n_tok, device=dev) for h in range(H)}
            V = {h: synth.draw_v(seed, 0, h, 0, n_tok, device=dev) for h in range(H)}
            p = 0
            while p < S:
                n = min(rng.choice([C, C, max(1, C // 2), max(1, C - 7)]), S - p)
                for h0, nh in calls:
                    hs = range(h0, h0 + nh)
                    out = torch.empty(nh, G, n, 128, dtype=torch.float32, device=dev)
                    ss.prefill_group(0, h0, nh, torch.stack([Q[h][:, p:p + n] for h in hs]).contiguous(),
                                     torch.stack([K[h][p:p + n] for h in hs]).contiguous(),
                                     torch.stack([V[h][p:p + n] for h in hs]).contiguous(), p, out)
                    for i, h in enumerate(hs):
                        pre[h].append(out[i])
                p += n
            for t in range(nd):
                p = S + t
                for h0, nh in calls:
                    hs = range(h0, h0 + nh)
                    out = torch.empty(nh, G, 128, dtype=torch.float32, device=dev)
                    ss.decode_group(0, h0, nh, torch.stack([Q[h][:, p] for h in hs]).contiguous(),
                                    torch.stack([K[h][p] for h in hs]).contiguous(),
                                    torch.stack([V[h][p] for h in hs]).contiguous(), p, out)
                    for i, h in enumerate(hs):
                        dec[h].append(out[i])
        ss.sync()
    for h in range(H):
        q, k, v = synth.to_f64(Q[h].cpu()) / qs, synth.to_f64(K[h].cpu()), synth.to_f64(V[h].cpu())
        ref = os_.attn_head_streaming(q, k, v, 0, n_sink, n_recent) if h >= n_ret else oa.attn_head(q, k, v)
        got = torch.cat(pre[h], dim=1).cpu()
        for g in range(G):
            check(got[g], ref[g, :S], f"{c} prefill head {h} q {g}")
            if nd:
                check(torch.stack(dec[h], dim=1).cpu()[g], ref[g, S:], f"{c} decode head {h} q {g}")
