"""Head groups (Section 4, adaptive head-wise offloading): several KV heads per call give the same results as one
head per call, element by element against the fp64 oracle, in both modes, for prefill and decode."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
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


def run(mode, H, G, S, C, n_decode, group, seed, flags=0):
    """Chunked prefill then decode steps of one layer with `group` heads per call; returns outputs per head."""
    dev = "cuda:0"
    n_tok = S + n_decode
    with Session(1, H, G, n_tok, C, mode=mode, out_fp32=1) as ss:
        if flags:
            hb.hi_ctx_set_flags(ss.ctx, flags)
        if mode == hb.HI_MODE_OFFLOAD:        # any read of a row that was never fetched or written shows up as NaN
            ss.staging.view(torch.int16).fill_(0x7FC1)
            ss.kv.view(torch.int16).fill_(0x7FC1)
        pre = [[] for _ in range(H)]
        dec = [[] for _ in range(H)]
        with torch.cuda.stream(ss.s_compute):
            Q = torch.stack([synth.draw_q(seed, 0, a, 0, n_tok, device=dev) for a in range(H * G)]).view(H, G, n_tok, 128)
            K = torch.stack([synth.draw_k(seed, 0, h, 0, n_tok, device=dev) for h in range(H)])
            V = torch.stack([synth.draw_v(seed, 0, h, 0, n_tok, device=dev) for h in range(H)])
            units = []
            for p in range(0, S, C):
                for h0 in range(0, H, group):
                    units.append((p, min(C, S - p), h0, min(group, H - h0)))
            for u, (p, n, h0, nh) in enumerate(units):
                q = Q[h0:h0 + nh, :, p:p + n].contiguous()
                k = K[h0:h0 + nh, p:p + n].contiguous()
                v = V[h0:h0 + nh, p:p + n].contiguous()
                out = torch.empty(nh, G, n, 128, dtype=torch.float32, device=dev)
                nxt = None
                if u + 1 < len(units):
                    np_, _, nh0, nnh = units[u + 1]
                    nxt = (0, nh0, nnh, np_)
                ss.prefill_group(0, h0, nh, q, k, v, p, out, nxt)
                for j in range(nh):
                    pre[h0 + j].append(out[j])
            for t in range(n_decode):
                p = S + t
                for h0 in range(0, H, group):
                    nh = min(group, H - h0)
                    q = Q[h0:h0 + nh, :, p].contiguous()
                    k = K[h0:h0 + nh, p].contiguous()
                    v = V[h0:h0 + nh, p].contiguous()
                    out = torch.empty(nh, G, 128, dtype=torch.float32, device=dev)
                    ss.decode_group(0, h0, nh, q, k, v, p, out, None)
                    for j in range(nh):
                        dec[h0 + j].append(out[j])
        ss.sync()
        cache = ss.cache_view()[0].to("cpu").clone()          # [H][2][S_max][128]
        stats = ss.stats()
    pre = [torch.cat(x, dim=1).cpu() for x in pre]
    dec = [torch.stack(x, dim=1).cpu() for x in dec] if n_decode else None
    return pre, dec, cache, Q.cpu(), K.cpu(), V.cpu(), stats


@pytest.mark.parametrize("mode", [hb.HI_MODE_RESIDENT, hb.HI_MODE_OFFLOAD])
@pytest.mark.parametrize("group", [2, 3, 4])
def test_groups_match_oracle_and_single_head_calls(mode, group):
    H, G, S, C, nd, seed = 4, 4, 1350, 200, 3, 6100
    pre, dec, cache, Q, K, V, stats = run(mode, H, G, S, C, nd, group, seed)
    pre1, dec1, cache1, *_ = run(mode, H, G, S, C, nd, 1, seed)
    assert torch.equal(cache, cache1)
    for h in range(H):
        ref = oa.attn_head(synth.to_f64(Q[h]), synth.to_f64(K[h]), synth.to_f64(V[h]))     # [G][S+nd][128]
        for g in range(G):
            check(pre[h][g], ref[g, :S], f"prefill group {group} head {h} q {g}")
            check(dec[h][g], ref[g, S:], f"decode group {group} head {h} q {g}")
        # the grouping only changes where the rows are cut into slices and splits (hence which bf16 roundings of
        # the probabilities meet), not the result
        assert (pre[h] - pre1[h]).abs().max() < 4e-3
        assert (dec[h] - dec1[h]).abs().max() < 4e-3
        assert torch.equal(cache[h, 0, :S + nd], K[h]) and torch.equal(cache[h, 1, :S + nd], V[h])


@pytest.mark.parametrize("mode", [hb.HI_MODE_RESIDENT, hb.HI_MODE_OFFLOAD])
def test_all_heads_in_one_group_with_the_8wave_kernel(mode):
    # group of all 8 heads = layer-wise granularity; forced 8-wave kernel (split-KV over a group launch)
    H, G, S, C, seed = 8, 4, 4700, 520, 6200
    pre, _, cache, Q, K, V, stats = run(mode, H, G, S, C, 0, 8, seed, flags=hb.HI_FLAG_PREFILL_DEEP)
    for h in (0, 3, 7):
        ref = oa.attn_head(synth.to_f64(Q[h]), synth.to_f64(K[h]), synth.to_f64(V[h]))
        for g in range(G):
            check(pre[h][g], ref[g], f"8-head group, head {h} q {g}")
    if mode == hb.HI_MODE_OFFLOAD:
        assert stats.peak_staging_bytes <= (S * 512)      # still at most one head's worth of K/V in HBM


def test_group_argument_errors():
    with Session(1, 4, 4, 512, 64, mode=hb.HI_MODE_OFFLOAD, out_fp32=1) as ss:
        dev = "cuda:0"
        q = torch.zeros(4, 4, 64, 128, dtype=torch.bfloat16, device=dev)
        k = torch.zeros(4, 64, 128, dtype=torch.bfloat16, device=dev)
        out = torch.zeros(4, 4, 64, 128, dtype=torch.float32, device=dev)
        assert hb.hi_prefill_group(ss.ctx, 0, 2, 3, q, k, k, 0, 64, out, check=False) == hb.HI_ERR_ARG      # heads 2..4
        assert hb.hi_prefill_group(ss.ctx, 0, 0, 0, q, k, k, 0, 64, out, check=False) == hb.HI_ERR_ARG
        # 512-token budget -> 128-row slices: 4 heads x 64 rows do not fit
        assert ss.plan.slice_tokens == 128
        assert hb.hi_prefill_group(ss.ctx, 0, 0, 4, q, k, k, 0, 64, out, check=False) == hb.HI_ERR_HBM_BUDGET
        assert hb.hi_prefill_group(ss.ctx, 0, 0, 2, q, k, k, 0, 64, out, -1, 0, 1, 0, check=False) == hb.HI_OK
        ss.sync()


@pytest.mark.parametrize("mode", [hb.HI_MODE_OFFLOAD, hb.HI_MODE_RESIDENT])
def test_a_batch_of_ragged_sequences_is_more_heads(mode):
    """Eq. 4 has a batch dimension; for attention a batch element is just more KV heads with their own cache rows.
    Three sequences of different lengths x 2 KV heads as a 6-head layer: each sequence is prefilled and decoded at
    its own positions (two heads per call), interleaved token by token, and every head matches the oracle."""
    Hs, G, C, nd, seed, dev = 2, 4, 128, 3, 6400, "cuda:0"
    lens = [700, 45, 333]                                  # prompt lengths of the batch
    B = len(lens)
    H = B * Hs
    with Session(1, H, G, max(lens) + nd, C, mode=mode, out_fp32=1) as ss:
        if mode == hb.HI_MODE_OFFLOAD:
            ss.staging.view(torch.int16).fill_(0x7FC1)
            ss.kv.view(torch.int16).fill_(0x7FC1)
        Q, K, V, pre, dec = {}, {}, {}, {}, {}
        with torch.cuda.stream(ss.s_compute):
            for b, S in enumerate(lens):
                for j in range(Hs):
                    h = b * Hs + j
                    Q[h] = torch.stack([synth.draw_q(seed, 0, h * G + g, 0, S + nd, device=dev) for g in range(G)])
                    K[h] = synth.draw_k(seed, 0, h, 0, S + nd, device=dev)
                    V[h] = synth.draw_v(seed, 0, h, 0, S + nd, device=dev)
                    pre[h], dec[h] = [], []
            # prefill: chunk by chunk over the batch; a sequence that has run out of prompt sits the chunk out
            for p in range(0, max(lens), C):
                for b, S in enumerate(lens):
                    n = min(C, S - p)
                    if n <= 0:
                        continue
                    hs = range(b * Hs, (b + 1) * Hs)
                    out = torch.empty(Hs, G, n, 128, dtype=torch.float32, device=dev)
                    ss.prefill_group(0, b * Hs, Hs, torch.stack([Q[h][:, p:p + n] for h in hs]).contiguous(),
                                     torch.stack([K[h][p:p + n] for h in hs]).contiguous(),
                                     torch.stack([V[h][p:p + n] for h in hs]).contiguous(), p, out)
                    for i, h in enumerate(hs):
                        pre[h].append(out[i])
            for t in range(nd):
                for b, S in enumerate(lens):
                    hs = range(b * Hs, (b + 1) * Hs)
                    out = torch.empty(Hs, G, 128, dtype=torch.float32, device=dev)
                    nb = (b + 1) % B
                    nxt = (0, nb * Hs, Hs, lens[nb] + t + (1 if nb == 0 else 0))
                    ss.decode_group(0, b * Hs, Hs, torch.stack([Q[h][:, S + t] for h in hs]).contiguous(),
                                    torch.stack([K[h][S + t] for h in hs]).contiguous(),
                                    torch.stack([V[h][S + t] for h in hs]).contiguous(), S + t, out, nxt)
                    for i, h in enumerate(hs):
                        dec[h].append(out[i])
        ss.sync()
    for b, S in enumerate(lens):
        for j in range(Hs):
            h = b * Hs + j
            ref = oa.attn_head(synth.to_f64(Q[h].cpu()), synth.to_f64(K[h].cpu()), synth.to_f64(V[h].cpu()))
            check(torch.cat(pre[h], dim=1), ref[:, :S], f"sequence {b} head {j} prefill")
            check(torch.stack(dec[h], dim=1), ref[:, S:], f"sequence {b} head {j} decode")


def test_one_decode_launch_over_heads_of_different_lengths():
    """A batch of sequences of different lengths in HBM-resident heads: hi_decode_group_ragged serves all heads of all
    sequences in one split-KV launch and one combine launch, each head reading its own number of rows and appending
    its token's row at its own position.  Every head matches the oracle and the per-sequence calls."""
    Hs, G, nd, seed, dev = 2, 4, 3, 6500, "cuda:0"
    lens = [5000, 0, 45, 1333, 64]                         # rows already cached per sequence (one has none yet)
    B = len(lens)
    H = B * Hs
    S_max = max(lens) + nd
    with Session(1, H, G, S_max, 64, mode=hb.HI_MODE_RESIDENT, out_fp32=1) as ss, \
            Session(1, H, G, S_max, 64, mode=hb.HI_MODE_RESIDENT, out_fp32=1) as ref_ss:
        Q, K, V = {}, {}, {}
        with torch.cuda.stream(ss.s_compute):
            for h in range(H):
                n = lens[h // Hs] + nd
                Q[h] = torch.stack([synth.draw_q(seed, 0, h * G + g, 0, n, device=dev) for g in range(G)])
                K[h] = synth.draw_k(seed, 0, h, 0, n, device=dev)
                V[h] = synth.draw_v(seed, 0, h, 0, n, device=dev)
                for s_ in (ss, ref_ss):
                    cv = s_.cache_view()
                    cv[0, h, 0, :lens[h // Hs]].copy_(K[h][:lens[h // Hs]])
                    cv[0, h, 1, :lens[h // Hs]].copy_(V[h][:lens[h // Hs]])
            torch.cuda.synchronize()
            got, sep = [], []
            for t in range(nd):
                past = [lens[h // Hs] + t for h in range(H)]
                q = torch.stack([Q[h][:, past[h]] for h in range(H)]).contiguous()
                k = torch.stack([K[h][past[h]] for h in range(H)]).contiguous()
                v = torch.stack([V[h][past[h]] for h in range(H)]).contiguous()
                out = torch.empty(H, G, 128, dtype=torch.float32, device=dev)
                hb.hi_decode_group_ragged(ss.ctx, 0, 0, H, q, k, v, past, out)
                got.append(out)
                out2 = torch.empty(H, G, 128, dtype=torch.float32, device=dev)
                with torch.cuda.stream(ref_ss.s_compute):
                    for b in range(B):
                        ref_ss.decode_group(0, b * Hs, Hs, q[b * Hs:(b + 1) * Hs], k[b * Hs:(b + 1) * Hs],
                                            v[b * Hs:(b + 1) * Hs], lens[b] + t, out2[b * Hs:(b + 1) * Hs])
                sep.append(out2)
        ss.sync()
        ref_ss.sync()
        torch.cuda.synchronize()
        for h in range(H):
            n = lens[h // Hs]
            qf, kf, vf = synth.to_f64(Q[h].cpu()), synth.to_f64(K[h].cpu()), synth.to_f64(V[h].cpu())
            for t in range(nd):
                want = np.stack([oa.attn_rows(qf[g][n + t][None], kf, vf, np.array([n + t]))[0] for g in range(G)])
                check(got[t][h], want, f"ragged decode head {h} token {t}")
                assert (got[t][h] - sep[t][h]).abs().max() < 1e-3     # other partitions: bf16 rounding of the weights differs
            # the token rows were appended at each head's own position; nothing beyond was touched
            cv = ss.cache_view()[0, h].cpu()
            assert torch.equal(cv[0, :n + nd], K[h].cpu()) and torch.equal(cv[1, :n + nd], V[h].cpu())
    # offloaded heads share staging slices of one length: refused before anything is enqueued
    with Session(1, 2, G, 1024, 64, mode=hb.HI_MODE_OFFLOAD, out_fp32=1) as so:
        z = torch.zeros(2, G, 128, dtype=torch.bfloat16, device=dev)
        o = torch.zeros(2, G, 128, dtype=torch.float32, device=dev)
        assert hb.hi_decode_group_ragged(so.ctx, 0, 0, 2, z, z[:, 0], z[:, 0], [5, 9], o, check=False) == hb.HI_ERR_UNSUPPORTED
        assert hb.hi_decode_group_ragged(so.ctx, 0, 0, 2, z, z[:, 0], z[:, 0], [5, -1], o, check=False) == hb.HI_ERR_ARG
