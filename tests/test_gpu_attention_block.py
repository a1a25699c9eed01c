"""A whole attention block (projection + rotary embedding, head-wise attention with retrieval and streaming heads,
output projection) over several chunks and decode tokens: each stage against its oracle on the bits the stage
before it produced, and the composition against the oracle chain."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import projection as op
from oracle import streaming as os_
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import synth
from paper_2502_12574_amd.attention_block import AttentionBlock
from paper_2502_12574_amd.session import Session

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_round(a):
    return synth.to_f64(torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16))


@pytest.mark.parametrize("pre", [False, True])
@pytest.mark.parametrize("mode,T", [(hb.HI_MODE_OFFLOAD, 0), (hb.HI_MODE_OFFLOAD, 2), (hb.HI_MODE_RESIDENT, 1)])
def test_attention_block_prefill_and_decode(mode, T, pre):
    """pre: the block folds the softmax scale into the query projection (Session q_prescaled) - the oracle chain then
    rounds the scaled queries to bf16, as the projection does, and attends with them divided by the constant again."""
    D, Hkv, G, C, S, nd, theta, seed = 512, 4, 2, 256, 600, 4, 500000.0, 9400 + T
    Hq, n_sink, n_recent = Hkv * G, 6, 150
    n_tok = S + nd
    X = synth.draw_hidden(seed, 0, 0, n_tok, D, device=DEV)
    W = synth.draw_weight(seed, synth.TENSOR_WQKV, 0, (Hq + 2 * Hkv) * 128, D, device=DEV)
    Wo = synth.draw_weight(seed, synth.TENSOR_WO, 0, D, Hq * 128, device=DEV)
    Y = torch.full((n_tok, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    with Session(1, Hkv, G, 1024, C, mode=mode, out_fp32=0, streaming_heads=T, sink_tokens=n_sink,
                 recent_tokens=n_recent, q_prescaled=pre) as ss:
        blk = AttentionBlock(ss, 0, W, Wo, theta)
        for p in range(0, S, C):
            n = min(C, S - p)
            blk.forward(X[p:p + n], p, Y[p:p + n])
        for t in range(S, n_tok):
            blk.forward(X[t:t + 1], t, Y[t:t + 1])
        ss.sync()
        torch.cuda.synchronize()
        cache = ss.cache_view().to("cpu")

    # the oracle chain, rounding to bf16 where the GPU path stores bf16 (after the projection, after attention)
    Wf = synth.to_f64(W.cpu())
    Q, K, V = op.qkv_rope(synth.to_f64(X.cpu()), Wf[:Hq * 128], Wf[Hq * 128:(Hq + Hkv) * 128], Wf[(Hq + Hkv) * 128:],
                          np.arange(n_tok), 128, theta)
    if pre:
        Q = bf16_round(Q * hb.HI_Q_PRESCALE) / hb.HI_Q_PRESCALE
    else:
        Q = bf16_round(Q)
    K, V = bf16_round(K), bf16_round(V)
    A = np.empty((Hq, n_tok, 128))
    for h in range(Hkv):
        if h >= Hkv - T:
            A[h * G:(h + 1) * G] = os_.attn_head_streaming(Q[h * G:(h + 1) * G], K[h], V[h], 0, n_sink, n_recent)
        else:
            A[h * G:(h + 1) * G] = oa.attn_head(Q[h * G:(h + 1) * G], K[h], V[h])
    ref = op.out_proj(bf16_round(A), synth.to_f64(Wo.cpu()))
    got = synth.to_f64(Y.cpu())
    assert np.isfinite(got).all()
    # three bf16 roundings and the attention's own tolerance propagate through W_o (unit-variance rows)
    err = np.abs(got - ref).max()
    rel = np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum())
    assert err <= 5e-2 and rel <= 1e-2, (err, rel)
    # the K/V the projection produced are what the cache holds for the retrieval heads (bit for bit after rounding)
    for h in range(Hkv - T):
        k_gpu = synth.to_f64(cache[0, h, 0, :n_tok])
        assert np.abs(k_gpu - K[h]).max() <= 2.0 ** -6          # a bf16 ulp at |x| < 4: rounding of nearly equal fp32 values
        assert (k_gpu == K[h]).mean() > 0.99
