"""The steps either side of the attention calls: Q/K/V projection with rotary embedding into head-major layout
(Eq. 1) and the output projection of the concatenated heads (Eq. 9), GPU against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import projection as op
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import synth
from paper_2502_12574_amd.session import Session

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def close(got, ref, atol, rel_l2, what):
    got = got.detach().to("cpu").to(torch.float64).numpy()
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    err = float(np.abs(got - ref).max())
    rel = float(np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()))
    assert err <= atol and rel <= rel_l2, (what, err, rel)


def qkv_on_gpu(X, W, D, Hq, Hkv, C, past, theta, out_fp32):
    dt = torch.float32 if out_fp32 else torch.bfloat16
    q = torch.full((Hq, C, 128), float("nan"), dtype=dt, device=DEV)
    k = torch.full((Hkv, C, 128), float("nan"), dtype=dt, device=DEV)
    v = torch.full((Hkv, C, 128), float("nan"), dtype=dt, device=DEV)
    ws = torch.empty(hb.hi_proj_workspace_bytes(C), dtype=torch.uint8, device=DEV)
    s = torch.cuda.current_stream()
    hb.hi_qkv_rope(s, X, W, D, Hq, Hkv, C, past, theta, out_fp32, q, k, v, ws)
    torch.cuda.synchronize()
    return q, k, v


@pytest.mark.parametrize("D,Hq,Hkv,C,past,theta", [
    (256, 4, 2, 300, 12345, 500000.0),        # ragged token tile, two heads per weight tile
    (128, 3, 1, 64, 0, 10000.0),              # odd number of heads: the last weight tile is half empty
    (512, 2, 2, 1, 999, 500000.0),            # one token (decode)
    (256, 4, 4, 257, 77, 0.0),                # no rotation
    (4096, 32, 8, 700, 1048576 - 700, 500000.0),   # Llama-3-8B shapes at the end of a 1M-token context
])
def test_qkv_projection_with_rotary_embedding(D, Hq, Hkv, C, past, theta):
    seed = 9100 + D + C
    X = synth.draw_hidden(seed, 0, past, C, D, device=DEV)
    W = synth.draw_weight(seed, synth.TENSOR_WQKV, 0, (Hq + 2 * Hkv) * 128, D, device=DEV)
    Wf = synth.to_f64(W.cpu())
    Qr, Kr, Vr = op.qkv_rope(synth.to_f64(X.cpu()), Wf[:Hq * 128], Wf[Hq * 128:(Hq + Hkv) * 128],
                             Wf[(Hq + Hkv) * 128:], np.arange(past, past + C), 128, theta if theta > 0 else None)
    q32, k32, v32 = qkv_on_gpu(X, W, D, Hq, Hkv, C, past, theta, 1)
    # fp32 accumulation of D products of bf16 values, fp32 rotation with a double-precision angle
    for got, ref, what in ((q32, Qr, "Q"), (k32, Kr, "K"), (v32, Vr, "V")):
        close(got, ref, 2e-4, 2e-5, what)
    q16, k16, v16 = qkv_on_gpu(X, W, D, Hq, Hkv, C, past, theta, 0)
    for a16, a32 in ((q16, q32), (k16, k32), (v16, v32)):      # bf16 output = the fp32 output rounded to nearest even
        assert torch.equal(a16, a32.to(torch.bfloat16))


@pytest.mark.parametrize("D,Hq,C", [(256, 2, 300), (192, 3, 1), (4096, 32, 700)])
def test_output_projection_of_concatenated_heads(D, Hq, C):
    seed = 9200 + D + C
    A = torch.stack([synth.draw_q(seed, 0, h, 0, C, device=DEV) for h in range(Hq)])     # [Hq][C][128]
    W = synth.draw_weight(seed, synth.TENSOR_WO, 0, D, Hq * 128, device=DEV)
    ref = op.out_proj(synth.to_f64(A.cpu()), synth.to_f64(W.cpu()))
    y32 = torch.full((C, D), float("nan"), dtype=torch.float32, device=DEV)
    y16 = torch.full((C, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    s = torch.cuda.current_stream()
    hb.hi_out_proj(s, A, W, Hq, D, C, 1, y32)
    hb.hi_out_proj(s, A, W, Hq, D, C, 0, y16)
    torch.cuda.synchronize()
    close(y32, ref, 2e-4, 2e-5, "Y")
    assert torch.equal(y16, y32.to(torch.bfloat16))


def test_projection_attention_projection_chain():
    """hidden states -> hi_qkv_rope -> hi_prefill_group over all heads -> hi_out_proj, each stage checked against the
    oracle on the bits the previous stage produced (the layouts connect without any reshuffling)."""
    D, Hq, Hkv, G, C, past, theta, seed = 512, 4, 2, 2, 384, 0, 500000.0, 9300
    X = synth.draw_hidden(seed, 0, past, C, D, device=DEV)
    W = synth.draw_weight(seed, synth.TENSOR_WQKV, 0, (Hq + 2 * Hkv) * 128, D, device=DEV)
    Wo = synth.draw_weight(seed, synth.TENSOR_WO, 0, D, Hq * 128, device=DEV)
    q, k, v = qkv_on_gpu(X, W, D, Hq, Hkv, C, past, theta, 0)
    with Session(1, Hkv, G, 1024, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=0) as ss:
        attn = torch.empty(Hkv, G, C, 128, dtype=torch.bfloat16, device=DEV)
        with torch.cuda.stream(ss.s_compute):
            ss.prefill_group(0, 0, Hkv, q.view(Hkv, G, C, 128), k, v, 0, attn)
        ss.sync()
        y = torch.empty(C, D, dtype=torch.float32, device=DEV)
        hb.hi_out_proj(ss.s_compute, attn, Wo, Hq, D, C, 1, y)
        ss.sync()
    ref_attn = oa.attn_layer(synth.to_f64(q.cpu()), synth.to_f64(k.cpu()), synth.to_f64(v.cpu()))
    close(attn.view(Hq, C, 128), ref_attn, 1.6e-2, 5e-3, "attention on the projected heads")
    close(y, op.out_proj(synth.to_f64(attn.view(Hq, C, 128).cpu()), synth.to_f64(Wo.cpu())), 2e-4, 2e-5, "Y")


def test_projection_argument_errors():
    x = torch.zeros(8, 256, dtype=torch.bfloat16, device=DEV)
    w = torch.zeros(3 * 128, 256, dtype=torch.bfloat16, device=DEV)
    o = torch.zeros(1, 8, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(hb.hi_proj_workspace_bytes(8), dtype=torch.uint8, device=DEV)
    s = torch.cuda.current_stream()
    assert hb.hi_qkv_rope(s, x, w, 200, 1, 1, 8, 0, 1e4, 0, o, o, o, ws, check=False) == hb.HI_ERR_UNSUPPORTED
    assert hb.hi_qkv_rope(s, x, w, 256, 1, 1, 0, 0, 1e4, 0, o, o, o, ws, check=False) == hb.HI_ERR_ARG
    assert hb.hi_qkv_rope(s, x, w, 256, 1, 1, 8, 0, 1e4, 0, o, o, o, None, check=False) == hb.HI_ERR_ARG
    assert hb.hi_qkv_rope(s, None, w, 256, 1, 1, 8, 0, 1e4, 0, o, o, o, ws, check=False) == hb.HI_ERR_ARG
    assert hb.hi_out_proj(s, o, w, 0, 256, 8, 0, x, check=False) == hb.HI_ERR_ARG
    torch.cuda.synchronize()


@pytest.mark.parametrize("case_id", range(16))
def test_projection_random_shapes(case_id):
    import random
    rng = random.Random(9500 + case_id)
    D = rng.choice([128, 256, 384, 640, 1024])
    Hq, Hkv = rng.randint(1, 6), rng.randint(1, 3)
    C = rng.choice([1, 2, 31, 255, 256, 257, rng.randint(1, 700)])
    past = rng.choice([0, 5, 99999, 4000000])
    theta = rng.choice([0.0, 10000.0, 500000.0])
    seed = 9500 + case_id
    X = synth.draw_hidden(seed, 0, past, C, D, device=DEV)
    W = synth.draw_weight(seed, synth.TENSOR_WQKV, 0, (Hq + 2 * Hkv) * 128, D, device=DEV)
    Wf = synth.to_f64(W.cpu())
    Qr, Kr, Vr = op.qkv_rope(synth.to_f64(X.cpu()), Wf[:Hq * 128], Wf[Hq * 128:(Hq + Hkv) * 128],
                             Wf[(Hq + Hkv) * 128:], np.arange(past, past + C), 128, theta if theta > 0 else None)
    q, k, v = qkv_on_gpu(X, W, D, Hq, Hkv, C, past, theta, 1)
    what = f"D={D} Hq={Hq} Hkv={Hkv} C={C} past={past} theta={theta}"
    for got, ref, name in ((q, Qr, "Q"), (k, Kr, "K"), (v, Vr, "V")):
        close(got, ref, 2e-4, 2e-5, f"{name} {what}")
    Dm = rng.choice([128, 200, 256, 777])            # the output width need not be a multiple of anything
    A = torch.stack([synth.draw_q(seed, 0, h, 0, C, device=DEV) for h in range(Hq)])
    Wo = synth.draw_weight(seed, synth.TENSOR_WO, 0, Dm, Hq * 128, device=DEV)
    y = torch.full((C, Dm), float("nan"), dtype=torch.float32, device=DEV)
    hb.hi_out_proj(torch.cuda.current_stream(), A, Wo, Hq, Dm, C, 1, y)
    torch.cuda.synchronize()
    close(y, op.out_proj(synth.to_f64(A.cpu()), synth.to_f64(Wo.cpu())), 2e-4, 2e-5, f"Y Dm={Dm} {what}")
