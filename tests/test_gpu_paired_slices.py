"""Short staging slices reach the 16x16x32 prefill kernels two at a time (one launch over two ring slots, the second
slot's rows behind a jump inside the past segment).  Chunked prefill of two offloaded heads with slices of 24 tiles,
so that units have one, two, three and four slices, pairs start at even and odd ring slots and wrap around the ring;
every output row against the oracle, and the launch counts against the same run with one launch per slice."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2502_12574_amd import binding as hb
from paper_2502_12574_amd import synth
from paper_2502_12574_amd.session import Session

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, REL_L2 = 1e-2, 5e-3
FORMS = {"eight-wave": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_8WAVE,
         "wide": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_WIDE,
         "wide, balanced triangle": hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_WIDE | hb.HI_FLAG_PREFILL_PAIRED}


def run(flags, seed, H, G, S, C, pre, link_kv_bits=0):
    qs = hb.HI_Q_PRESCALE if pre else 1.0
    outs = {h: [] for h in range(H)}
    with Session(1, H, G, S, C, mode=hb.HI_MODE_OFFLOAD, out_fp32=1, q_prescaled=pre, link_kv_bits=link_kv_bits) as ss:
        hb.hi_ctx_set_flags(ss.ctx, flags)
        st = ss.plan.slice_tokens
        with torch.cuda.stream(ss.s_compute):
            Q = {h: torch.stack([synth.draw_q(seed, 0, h * G + g, 0, S, device=DEV, scale=qs) for g in range(G)])
                 for h in range(H)}
            K = {h: synth.draw_k(seed, 0, h, 0, S, device=DEV, peaked=True) for h in range(H)}
            V = {h: synth.draw_v(seed, 0, h, 0, S, device=DEV) for h in range(H)}
            for p in range(0, S, C):
                n = min(C, S - p)
                for h in range(H):
                    out = torch.empty(G, n, 128, dtype=torch.float32, device=DEV)
                    nxt = (0, h + 1, p) if h + 1 < H else (0, 0, p + n)
                    ss.prefill_head(0, h, Q[h][:, p:p + n].contiguous(), K[h][p:p + n], V[h][p:p + n], p, out, nxt)
                    outs[h].append(out)
        ss.sync()
        launches = ss.stats().n_prefill_kernels
    got = {h: torch.cat(outs[h], dim=1).cpu() for h in range(H)}
    return got, {h: Q[h].cpu() for h in range(H)}, {h: K[h].cpu() for h in range(H)}, {h: V[h].cpu() for h in range(H)}, \
        launches, st


@pytest.mark.parametrize("form", list(FORMS))
@pytest.mark.parametrize("pre", [True, False])
def test_pairs_of_slices(form, pre):
    seed, H, G, S, C = 41000, 2, 4, 6144, 512
    got, Q, K, V, launches, st = run(FORMS[form], seed, H, G, S, C, pre)
    _, _, _, _, launches_single, _ = run(FORMS[form] | hb.HI_FLAG_PREFILL_SINGLE_SLICES, seed, H, G, S, C, pre)
    assert st % 64 == 0 and 8 * 64 <= st < S // 3, st          # several slices per unit, steady-state runs in each
    n_slices = [-(-p // st) for p in range(0, S, C)]
    assert launches_single == H * sum(max(1, n) for n in n_slices)
    assert launches == H * sum(max(1, -(-n // 2)) for n in n_slices) and launches < launches_single
    qs = hb.HI_Q_PRESCALE if pre else 1.0
    for h in range(H):
        ref = oa.attn_head(synth.to_f64(Q[h]) / qs, synth.to_f64(K[h]), synth.to_f64(V[h]))
        g64 = got[h].double().numpy()
        assert np.isfinite(g64).all()
        err = float(np.abs(g64 - ref).max())
        rel = float(np.sqrt(((g64 - ref) ** 2).sum() / (ref ** 2).sum()))
        assert err <= MAX_ABS and rel <= REL_L2, (form, pre, h, err, rel)


def test_the_other_kernels_take_one_slice_per_launch():
    """The 32x32x16 form has no two-piece past segment: the library does not pair for it."""
    seed, H, G, S, C = 41001, 1, 4, 4096, 512
    f = hb.HI_FLAG_PREFILL_DEEP | hb.HI_FLAG_PREFILL_MFMA32
    _, _, _, _, launches, st = run(f, seed, H, G, S, C, False)
    assert launches == H * sum(max(1, -(-p // st)) for p in range(0, S, C))


@pytest.mark.parametrize("form", ["eight-wave", "wide"])
def test_a_ring_of_two_slots_is_not_paired(form):
    """With 4-bit rows on the link the plan's ring has two (larger) slots: a pair would be the whole ring and nothing
    could land under the kernel, so the library launches once per slice."""
    seed, H, G, S, C = 41002, 2, 4, 6144, 512
    got, _, _, _, launches, st = run(FORMS[form], seed, H, G, S, C, True, link_kv_bits=4)
    one, _, _, _, launches_single, _ = run(FORMS[form] | hb.HI_FLAG_PREFILL_SINGLE_SLICES, seed, H, G, S, C, True,
                                           link_kv_bits=4)
    assert launches == launches_single
    for h in range(H):
        assert torch.isfinite(got[h]).all() and torch.equal(got[h], one[h])
