"""GPU parity at the configurations' full sizes, in the launch configuration bench.py times (offloaded, one KV
head of HBM staging, driver loops with prefetch hints), on sampled outputs the fp64 oracle computes one by one.

Inputs are regenerated on the CPU by the seeded generator (integer-only, bit-identical to the GPU draw), so no
oracle input or expected value comes from the GPU path.  Tolerance as in the small tests: max-abs 1e-2 and
relative L2 5e-3 per (call, query head) on fp32 output.
"""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import driver, synth
from paper_2502_12574_amd.session import Session

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
MAX_ABS, REL_L2 = 1e-2, 5e-3
DEV = "cuda:0"


def cpu_f64(tensor_id, seed, layer, head, n, peaked=False, step=1 << 19):
    """float64 [n, 128] of one K/V/Q stream, drawn on the CPU in slices (bounded temporaries)."""
    out = np.empty((n, 128), dtype=np.float64)
    for a in range(0, n, step):
        b = min(n, a + step)
        if tensor_id == synth.TENSOR_K:
            t = synth.draw_k(seed, layer, head, a, b - a, peaked=peaked)
        else:
            t = synth.draw(seed, tensor_id, layer, head, a, b - a)
        out[a:b] = t.to(torch.float64).numpy()
    return out


def check_rows(got, ref, what):
    got = got.detach().to("cpu").to(torch.float64).numpy()
    assert np.isfinite(got).all(), what
    err = float(np.abs(got - ref).max())
    rel = float(np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()))
    assert err <= MAX_ABS and rel <= REL_L2, (what, err, rel)
    return err, rel


def sample_positions(S, C, slice_tokens, rng, n_random):
    pts = {0, 1, C - 1, C, C + 1, S - C - 1, S - C, S - C + 1, S - 2, S - 1, S // 2, S // 2 + 31, S // 2 + 32}
    for b in (slice_tokens, 2 * slice_tokens):
        if b < S:
            pts |= {b - 1, b, b + 1}
    pts |= set(int(x) for x in rng.integers(0, S, n_random))
    return np.array(sorted(p for p in pts if 0 <= p < S), dtype=np.int64)


def fill_host_cache(ss, seed, layer, heads, n_rows, peaked=False, step=1 << 18):
    """Pre-fill rows [0, n_rows) of the pinned cache with the synthetic K/V (drawn on the GPU, copied down)."""
    cv = ss.cache_view()
    for h in heads:
        for a in range(0, n_rows, step):
            b = min(n_rows, a + step)
            cv[layer, h, 0, a:b].copy_(synth.draw_k(seed, layer, h, a, b - a, device=DEV, peaked=peaked))
            cv[layer, h, 1, a:b].copy_(synth.draw_v(seed, layer, h, a, b - a, device=DEV))
    torch.cuda.synchronize()


def test_config2_128k_prefill_sampled_rows():
    """Llama-3-8B-shaped layer, 128K context, chunk 8192, 32 Q / 8 KV heads, offloaded head-wise chunked prefill."""
    seed, S, C, H, G = 20250214, 131072, 8192, 8, 4
    rng = np.random.default_rng(2)
    with Session(1, H, G, S, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=1) as ss:
        pos = sample_positions(S, C, ss.plan.slice_tokens, rng, 40)
        by_chunk = {}
        for p in pos:
            by_chunk.setdefault(int(p) // C, []).append(int(p) % C)
        kept = {}

        def keep(c, l, h, out):
            if c in by_chunk:
                idx = torch.tensor(by_chunk[c], device=DEV)
                kept[(c, h)] = out.index_select(1, idx)

        with torch.cuda.stream(ss.s_compute):
            inp = driver.LayerInputs(seed, 1, H, G, S, C, DEV)
            driver.prefill(ss, inp, keep=keep)
        ss.sync()
        st = ss.stats()
        assert st.peak_staging_bytes <= ss.plan.host_bytes_per_head
        assert st.bytes_h2d == 512 * H * sum(range(0, S, C)) and st.bytes_d2h == 512 * H * S
        worst = (0.0, 0.0)
        for h in range(H):
            K = cpu_f64(synth.TENSOR_K, seed, 0, h, S)
            V = cpu_f64(synth.TENSOR_V, seed, 0, h, S)
            # write-back exactness on sampled rows of the host cache
            cv = ss.cache_view()
            for p in pos[::7]:
                assert torch.equal(cv[0, h, 0, int(p)], synth.draw_k(seed, 0, h, int(p), 1)[0])
                assert torch.equal(cv[0, h, 1, int(p)], synth.draw_v(seed, 0, h, int(p), 1)[0])
            for g in range(G):
                qrows = synth.to_f64(torch.cat([synth.draw_q(seed, 0, h * G + g, int(p), 1) for p in pos]))
                ref = oa.attn_rows(qrows, K, V, pos)
                got = torch.cat([kept[(c, h)][g] for c in sorted(by_chunk)])
                e = check_rows(got, ref, f"cfg2 kv head {h} q head {g}")
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        print("config 2 worst (max-abs, rel-L2):", worst)


def test_config3_decode_1m_offloaded_and_resident():
    """Decode at a 1M-token context: K/V pre-filled in pinned host memory, streamed one KV head at a time through
    the one-head staging ring; the same steps with K/V resident in HBM."""
    seed, S, H, G, nd = 20250215, 1 << 20, 8, 4, 3
    checked = (0, 5)                      # KV heads compared with the oracle (CPU regeneration is the slow part)
    ss = Session(1, H, G, S + nd, 64, mode=hb.HI_MODE_OFFLOAD, out_fp32=1)
    fill_host_cache(ss, seed, 0, range(H), S)
    with torch.cuda.stream(ss.s_compute):
        inp = driver.LayerInputs(seed, 1, H, G, 64, 64, DEV)          # only its decode_rows() is used
        rows = [inp.decode_rows(S + t) for t in range(nd)]
        off = driver.decode(ss, inp, S, nd, rows=rows)
    ss.sync()
    st = ss.stats()
    assert st.peak_staging_bytes <= ss.plan.host_bytes_per_head
    assert st.bytes_h2d == 512 * H * sum(S + t for t in range(nd))
    rs = Session(1, H, G, S + nd, 64, mode=hb.HI_MODE_RESIDENT, out_fp32=1)
    rs.kv.copy_(ss.kv)
    # the resident copy must not contain the rows the offloaded run appended
    rs.cache_view()[0, :, :, S:].zero_()
    with torch.cuda.stream(rs.s_compute):
        res = driver.decode(rs, inp, S, nd, rows=rows)
    rs.sync()
    for t in range(nd):
        a, b = off[t].cpu(), res[t].cpu()
        assert torch.isfinite(a).all() and (a - b).abs().max() < 2e-5       # same math, different partitions
    # appended rows reached both caches
    for h in range(H):
        for t in range(nd):
            for which, draw in ((0, synth.draw_k), (1, synth.draw_v)):
                row = draw(seed, 0, h, S + t, 1)[0]
                assert torch.equal(ss.cache_view()[0, h, which, S + t], row)
                assert torch.equal(rs.cache_view()[0, h, which, S + t].cpu(), row)
    for h in checked:
        K = cpu_f64(synth.TENSOR_K, seed, 0, h, S + nd)
        V = cpu_f64(synth.TENSOR_V, seed, 0, h, S + nd)
        for t in range(nd):
            q = np.stack([synth.to_f64(synth.draw_q(seed, 0, h * G + g, S + t, 1))[0] for g in range(G)])
            ref = oa.attn_rows(q, K, V, np.full(G, S + t))
            for g in range(G):
                check_rows(off[t][0, h, g:g + 1], ref[g:g + 1], f"cfg3 offloaded head {h} step {t} q {g}")
                check_rows(res[t][0, h, g:g + 1], ref[g:g + 1], f"cfg3 resident head {h} step {t} q {g}")
    ss.close()
    rs.close()


def test_config4_layer_1m_prefill_tail_sampled_rows():
    """One layer of the 1M-token configuration (chunk 16384) in the benchmark's launch configuration.  The cache is
    pre-filled up to the last two chunks, which then run through the library (every unit streams ~1M past rows
    through the staging ring in 8 slices); sampled rows against the oracle, then two decode steps.  As in the
    benchmark, the queries carry the softmax scale (hi_problem.q_prescaled); the oracle gets them divided by it."""
    seed, S, C, H, G, nd = 20250216, 1 << 20, 16384, 8, 4, 2
    QS = hb.HI_Q_PRESCALE
    checked = (2,)
    P0 = S - 2 * C
    rng = np.random.default_rng(4)
    ss = Session(1, H, G, S + nd, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=1, q_prescaled=True)
    fill_host_cache(ss, seed, 0, range(H), P0)
    pos = np.array(sorted({P0, P0 + 1, P0 + 63, P0 + 64, S - C - 1, S - C, S - C + 1, S - 1, S - 2} |
                          set(int(x) for x in rng.integers(P0, S, 24))), dtype=np.int64)
    kept = {}
    with torch.cuda.stream(ss.s_compute):
        for ci, p in enumerate((P0, P0 + C)):
            for h in range(H):
                q = torch.stack([synth.draw_q(seed, 0, h * G + g, p, C, device=DEV, scale=QS) for g in range(G)])
                k = synth.draw_k(seed, 0, h, p, C, device=DEV)
                v = synth.draw_v(seed, 0, h, p, C, device=DEV)
                out = torch.empty(G, C, 128, dtype=torch.float32, device=DEV)
                nxt = (0, h + 1, p) if h + 1 < H else ((0, 0, p + C) if ci == 0 else (0, 0, S))
                ss.prefill_head(0, h, q, k, v, p, out, nxt)
                if h in checked:
                    sel = [int(x - p) for x in pos if p <= x < p + C]
                    kept[(ci, h)] = out.index_select(1, torch.tensor(sel, device=DEV))
        inp = driver.LayerInputs(seed, 1, H, G, 64, 64, DEV, q_scale=QS)
        rows = [inp.decode_rows(S + t) for t in range(nd)]
        dec = driver.decode(ss, inp, S, nd, rows=rows)
    ss.sync()
    assert ss.stats().peak_staging_bytes <= ss.plan.host_bytes_per_head
    for h in checked:
        K = cpu_f64(synth.TENSOR_K, seed, 0, h, S + nd)
        V = cpu_f64(synth.TENSOR_V, seed, 0, h, S + nd)
        for g in range(G):
            qrows = synth.to_f64(torch.cat([synth.draw_q(seed, 0, h * G + g, int(p), 1, scale=QS) for p in pos])) / QS
            ref = oa.attn_rows(qrows, K, V, pos)
            got = torch.cat([kept[(0, h)][g], kept[(1, h)][g]])
            print("config 4 head", h, g, check_rows(got, ref, f"cfg4 kv head {h} q head {g}"))
        for t in range(nd):
            q = np.stack([synth.to_f64(synth.draw_q(seed, 0, h * G + g, S + t, 1, scale=QS))[0] for g in range(G)]) / QS
            ref = oa.attn_rows(q, K, V, np.full(G, S + t))
            for g in range(G):
                check_rows(dec[t][0, h, g:g + 1], ref[g:g + 1], f"cfg4 decode head {h} step {t} q {g}")
    ss.close()


def test_config5_4m_peaked_keys_tail_and_decode():
    """Extreme context: 4M tokens, chunk 32768, one key row in ten scaled x4 (peaked softmax rows; row offsets
    beyond 2**31 bytes).  The cache is pre-filled up to the last chunk, which runs through the library for one KV
    head (16 staging slices), followed by one decode step; sampled rows against the oracle."""
    seed, S, C, H, G = 20250217, 1 << 22, 32768, 8, 4
    h = 6                                  # a head far into the cache: its K plane starts 12 GiB in
    P0 = S - C
    rng = np.random.default_rng(5)
    ss = Session(1, H, G, S + 1, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=1)
    assert ss.plan.host_bytes_total > (1 << 34)
    fill_host_cache(ss, seed, 0, [h], P0, peaked=True)
    pos = np.array(sorted({P0, P0 + 1, P0 + 31, P0 + 32, S - 1, S - 2} | set(int(x) for x in rng.integers(P0, S, 10))),
                   dtype=np.int64)
    with torch.cuda.stream(ss.s_compute):
        q = torch.stack([synth.draw_q(seed, 0, h * G + g, P0, C, device=DEV) for g in range(G)])
        k = synth.draw_k(seed, 0, h, P0, C, device=DEV, peaked=True)
        v = synth.draw_v(seed, 0, h, P0, C, device=DEV)
        out = torch.empty(G, C, 128, dtype=torch.float32, device=DEV)
        ss.prefill_head(0, h, q, k, v, P0, out, (0, h, S))
        got = out.index_select(1, torch.tensor([int(x - P0) for x in pos], device=DEV))
        qd = torch.stack([synth.draw_q(seed, 0, h * G + g, S, 1, device=DEV)[0] for g in range(G)])
        kd = synth.draw_k(seed, 0, h, S, 1, device=DEV, peaked=True)[0]
        vd = synth.draw_v(seed, 0, h, S, 1, device=DEV)[0]
        outd = torch.empty(G, 128, dtype=torch.float32, device=DEV)
        ss.decode_head(0, h, qd, kd, vd, S, outd)
    ss.sync()
    assert ss.stats().peak_staging_bytes <= ss.plan.host_bytes_per_head
    K = cpu_f64(synth.TENSOR_K, seed, 0, h, S + 1, peaked=True)
    V = cpu_f64(synth.TENSOR_V, seed, 0, h, S + 1)
    for g in range(G):
        qrows = synth.to_f64(torch.cat([synth.draw_q(seed, 0, h * G + g, int(p), 1) for p in pos]))
        ref = oa.attn_rows(qrows, K, V, pos)
        print("config 5 q head", g, check_rows(got[g], ref, f"cfg5 q head {g}"))
    ref = oa.attn_rows(synth.to_f64(qd), K, V, np.full(G, S))
    for g in range(G):
        check_rows(outd[g:g + 1], ref[g:g + 1], f"cfg5 decode q head {g}")
    ss.close()
