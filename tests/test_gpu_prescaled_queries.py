"""Queries that carry the softmax scale (hi_problem.q_prescaled): every attention kernel must compute the same function
of the model's q.  A pre-scaled query is HI_Q_PRESCALE = log2(e) / sqrt(128) times the q of Eq. 3, so the oracle is the
plain definition applied to q' / HI_Q_PRESCALE (an exact division in fp64): exp(q.k / sqrt(d)) = 2^(q'.k)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import projection as op
from oracle import streaming as os_
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import synth
from paper_2502_12574_amd.session import Session

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, REL_L2 = 1e-2, 5e-3
QS = hb.HI_Q_PRESCALE


def check(got, ref, what):
    got = got.detach().to("cpu").to(torch.float64).numpy()
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    err = float(np.abs(got - ref).max())
    rel = float(np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()))
    assert err <= MAX_ABS and rel <= REL_L2, (what, err, rel)


def test_the_constant():
    assert abs(QS - np.log2(np.e) / np.sqrt(128.0)) < 1e-15


@pytest.mark.parametrize("mode", [hb.HI_MODE_RESIDENT, hb.HI_MODE_OFFLOAD])
def test_chunked_prefill_and_decode(mode):
    seed, S, C, G, nd = 31001, 1500, 400, 4, 5
    with Session(1, 1, G, S + nd, C, mode=mode, out_fp32=1, q_prescaled=True) as ss:
        outs, dec = [], []
        with torch.cuda.stream(ss.s_compute):
            Q = torch.stack([synth.draw_q(seed, 0, g, 0, S + nd, device=DEV, scale=QS) for g in range(G)])
            K = synth.draw_k(seed, 0, 0, 0, S + nd, device=DEV)
            V = synth.draw_v(seed, 0, 0, 0, S + nd, device=DEV)
            for p in range(0, S, C):
                n = min(C, S - p)
                out = torch.empty(G, n, 128, dtype=torch.float32, device=DEV)
                ss.prefill_head(0, 0, Q[:, p:p + n].contiguous(), K[p:p + n], V[p:p + n], p, out, (0, 0, p + n))
                outs.append(out)
            for t in range(nd):
                p = S + t
                out = torch.empty(G, 128, dtype=torch.float32, device=DEV)
                ss.decode_head(0, 0, Q[:, p].contiguous(), K[p], V[p], p, out)
                dec.append(out)
        ss.sync()
    ref = oa.attn_head(synth.to_f64(Q.cpu()) / QS, synth.to_f64(K.cpu()), synth.to_f64(V.cpu()))
    got = torch.cat(outs, dim=1)
    for g in range(G):
        check(got[g], ref[g, :S], f"prefill head {g}")
        check(torch.stack(dec)[:, g], ref[g, S:], f"decode head {g}")


FORMS = {"default": 0, "deep": hb.HI_FLAG_PREFILL_DEEP, "wide": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_WIDE,
         "pairedwide": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_PAIRED | hb.HI_FLAG_PREFILL_WIDE, "deep32": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_MFMA32,
         "paired": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_PAIRED, "narrow": hb.HI_FLAG_PREFILL_NARROW}


@pytest.mark.parametrize("G,P,C", [(4, 0, 300), (4, 8000, 192), (1, 2100, 257), (8, 4200, 100), (2, 777, 512)])
@pytest.mark.parametrize("form", list(FORMS))
def test_every_prefill_kernel_form(G, P, C, form):
    """Pasts long enough for the steady-state loop (where the multiplication is compiled out), one key row in ten scaled
    x4 so that the running reference moves inside it."""
    seed = 31100 + P + C
    with Session(1, 1, G, max(P + C, 128), C, mode=hb.HI_MODE_RESIDENT, out_fp32=1, q_prescaled=True) as ss:
        hb.hi_ctx_set_flags(ss.ctx, FORMS[form])
        with torch.cuda.stream(ss.s_compute):
            Q = torch.stack([synth.draw_q(seed, 0, g, P, C, device=DEV, scale=QS) for g in range(G)])
            K = synth.draw_k(seed, 0, 0, 0, P + C, device=DEV, peaked=True)
            V = synth.draw_v(seed, 0, 0, 0, P + C, device=DEV)
            cv = ss.cache_view()
            if P:
                cv[0, 0, 0, :P].copy_(K[:P])
                cv[0, 0, 1, :P].copy_(V[:P])
            out = torch.empty(G, C, 128, dtype=torch.float32, device=DEV)
            ss.prefill_head(0, 0, Q, K[P:], V[P:], P, out)
        ss.sync()
    ref = oa.attn_head(synth.to_f64(Q.cpu()) / QS, synth.to_f64(K.cpu()), synth.to_f64(V.cpu()), past_len=P)
    for g in range(G):
        check(out[g], ref[g], f"{form} G={G} P={P} C={C} head {g}")


def test_prescaled_and_plain_queries_give_the_same_function():
    """The same model q handed over both ways (plain, and times the constant with one more rounding to bf16): the two
    outputs differ by what that rounding does to the scores, far inside the parity tolerance."""
    seed, G, P, C = 31200, 4, 3000, 256
    outs = []
    for pre in (False, True):
        with Session(1, 1, G, P + C, C, mode=hb.HI_MODE_RESIDENT, out_fp32=1, q_prescaled=pre) as ss:
            with torch.cuda.stream(ss.s_compute):
                Q = torch.stack([synth.draw_q(seed, 0, g, P, C, device=DEV, scale=QS if pre else 1.0) for g in range(G)])
                K = synth.draw_k(seed, 0, 0, 0, P + C, device=DEV)
                V = synth.draw_v(seed, 0, 0, 0, P + C, device=DEV)
                cv = ss.cache_view()
                cv[0, 0, 0, :P].copy_(K[:P])
                cv[0, 0, 1, :P].copy_(V[:P])
                out = torch.empty(G, C, 128, dtype=torch.float32, device=DEV)
                ss.prefill_head(0, 0, Q, K[P:], V[P:], P, out)
            ss.sync()
            outs.append(out.cpu())
    assert (outs[0] - outs[1]).abs().max() < 5e-3


def test_streaming_head_and_groups():
    """One retrieval pair called as a group and one streaming head, chunked prefill and decode, offloaded."""
    seed, H, G, S, C, nd, n_sink, n_recent = 31300, 3, 4, 900, 256, 3, 5, 100
    with Session(1, H, G, 1024, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=1, streaming_heads=1, sink_tokens=n_sink,
                 recent_tokens=n_recent, q_prescaled=True) as ss:
        pre = {h: [] for h in range(H)}
        dec = {h: [] for h in range(H)}
        with torch.cuda.stream(ss.s_compute):
            Q = {h: torch.stack([synth.draw_q(seed, 0, h * G + g, 0, S + nd, device=DEV, scale=QS) for g in range(G)])
                 for h in range(H)}
            K = {h: synth.draw_k(seed, 0, h, 0, S + nd, device=DEV) for h in range(H)}
            V = {h: synth.draw_v(seed, 0, h, 0, S + nd, device=DEV) for h in range(H)}
            for p in range(0, S, C):
                n = min(C, S - p)
                for h0, nh in ((0, 2), (2, 1)):
                    hs = range(h0, h0 + nh)
                    out = torch.empty(nh, G, n, 128, dtype=torch.float32, device=DEV)
                    ss.prefill_group(0, h0, nh, torch.stack([Q[h][:, p:p + n] for h in hs]).contiguous(),
                                     torch.stack([K[h][p:p + n] for h in hs]).contiguous(),
                                     torch.stack([V[h][p:p + n] for h in hs]).contiguous(), p, out)
                    for i, h in enumerate(hs):
                        pre[h].append(out[i])
            for t in range(nd):
                p = S + t
                for h0, nh in ((0, 2), (2, 1)):
                    hs = range(h0, h0 + nh)
                    out = torch.empty(nh, G, 128, dtype=torch.float32, device=DEV)
                    ss.decode_group(0, h0, nh, torch.stack([Q[h][:, p] for h in hs]).contiguous(),
                                    torch.stack([K[h][p] for h in hs]).contiguous(),
                                    torch.stack([V[h][p] for h in hs]).contiguous(), p, out)
                    for i, h in enumerate(hs):
                        dec[h].append(out[i])
        ss.sync()
    for h in range(H):
        q, k, v = synth.to_f64(Q[h].cpu()) / QS, synth.to_f64(K[h].cpu()), synth.to_f64(V[h].cpu())
        ref = os_.attn_head_streaming(q, k, v, 0, n_sink, n_recent) if h == 2 else oa.attn_head(q, k, v)
        got = torch.cat(pre[h], dim=1)
        for g in range(G):
            check(got[g], ref[g, :S], f"prefill head {h} q {g}")
            check(torch.stack(dec[h], dim=1)[g], ref[g, S:], f"decode head {h} q {g}")


@pytest.mark.parametrize("C", [300, 1])
def test_projection_folds_the_constant_into_the_query_heads_only(C):
    D, Hq, Hkv, past, theta, seed = 256, 4, 2, 4321, 500000.0, 31400
    X = synth.draw_hidden(seed, 0, past, C, D, device=DEV)
    W = synth.draw_weight(seed, synth.TENSOR_WQKV, 0, (Hq + 2 * Hkv) * 128, D, device=DEV)
    Wf = synth.to_f64(W.cpu())
    Qr, Kr, Vr = op.qkv_rope(synth.to_f64(X.cpu()), Wf[:Hq * 128], Wf[Hq * 128:(Hq + Hkv) * 128],
                             Wf[(Hq + Hkv) * 128:], np.arange(past, past + C), 128, theta)
    outs = {}
    for fp32 in (1, 0):
        dt = torch.float32 if fp32 else torch.bfloat16
        q = torch.full((Hq, C, 128), float("nan"), dtype=dt, device=DEV)
        k = torch.full((Hkv, C, 128), float("nan"), dtype=dt, device=DEV)
        v = torch.full((Hkv, C, 128), float("nan"), dtype=dt, device=DEV)
        ws = torch.empty(hb.hi_proj_workspace_bytes(C), dtype=torch.uint8, device=DEV)
        hb.hi_qkv_rope(torch.cuda.current_stream(), X, W, D, Hq, Hkv, C, past, theta, fp32, q, k, v, ws, q_scale=QS)
        torch.cuda.synchronize()
        outs[fp32] = (q, k, v)
    for got, ref, what in zip(outs[1], (Qr * QS, Kr, Vr), "QKV"):
        got = got.cpu().double().numpy()
        assert np.abs(got - ref).max() <= 2e-4 and np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()) <= 2e-5, what
    for a16, a32 in zip(outs[0], outs[1]):          # bf16 output = the scaled fp32 value rounded once
        assert torch.equal(a16, a32.to(torch.bfloat16))
    st = hb.hi_qkv_rope(torch.cuda.current_stream(), X, W, D, Hq, Hkv, C, past, theta, 0, *outs[0], ws, q_scale=0.0,
                        check=False)
    assert st == hb.HI_ERR_ARG
