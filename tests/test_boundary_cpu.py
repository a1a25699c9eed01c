"""CPU-only checks of the C-ABI boundary: the library loads, exports what the header declares, plans correctly
(against the memory-model oracle and the values the paper prints) and rejects bad arguments before any GPU call."""
import ctypes
import json
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import memory_model as mm
from paper_2502_12574_amd import binding as hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_memory_tables.json")))


def llama(S, C, **kw):
    return hb.make_problem(n_layers=32, n_kv_heads=8, gqa_group=4, max_context=S, chunk=C, **kw)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "headinfer.h")).read()
    code = re.sub(r"/\*.*?\*/", "", header, flags=re.S)            # declarations only, not the comments
    declared = set(re.findall(r"\b(hi_[a-z_]+)\s*\(", code))
    assert declared == set(hb.EXPORTS)
    raw = ctypes.CDLL(hb.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert hb.status_string(0) == "HI_OK" and hb.status_string(-5) == "HI_ERR_RANGE"


def test_struct_layouts_match_the_c_header(tmp_path):
    # compile the header with the host C compiler and compare sizes and a few offsets with the ctypes mirror
    src = tmp_path / "sz.c"
    src.write_text('''#include <stdio.h>
#include <stddef.h>
#include "headinfer.h"
int main(void){ printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(hi_problem), sizeof(hi_plan), sizeof(hi_stats),
  offsetof(hi_problem, mfma_TFLOPs), offsetof(hi_plan, regime_decode), offsetof(hi_stats, exposed_copy_ms)); return 0; }
''')
    exe = tmp_path / "sz"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    want = [ctypes.sizeof(hb.hi_problem), ctypes.sizeof(hb.hi_plan), ctypes.sizeof(hb.hi_stats),
            hb.hi_problem.mfma_TFLOPs.offset, hb.hi_plan.regime_decode.offset, hb.hi_stats.exposed_copy_ms.offset]
    assert got == want


def test_plan_pins_paper_memory_numbers():
    S = 1 << 20
    pl = hb.hi_offload_plan(llama(S, 16384))
    # Eq. 11: one head's K+V at 1M tokens = 512 MiB; Table 10 "1" GB is the two-head ping-pong
    assert pl.host_bytes_per_head == 512 << 20 == mm.head_bytes(mm.LLAMA3_8B, S)
    assert pl.hbm_pingpong_paper_bytes == 1 << 30
    assert pl.hbm_pingpong_paper_bytes / 2 ** 30 == GOLD["table10_1M_context"]["rows"]["headwise"]["kv"]
    # Eq. 4 / Table 10: 128 GB in total
    assert pl.host_bytes_total == 128 << 30 == mm.kv_cache_bytes(mm.LLAMA3_8B, S)
    assert pl.host_bytes_total / 2 ** 30 == GOLD["table10_1M_context"]["rows"]["headwise"]["total_kv"]
    # Eq. 10
    assert pl.alpha == GOLD["alpha"]["value"] == mm.alpha_headwise(mm.LLAMA3_8B)
    # the strict one-head budget: the ring never exceeds one head's bytes
    assert pl.hbm_staging_bytes <= pl.host_bytes_per_head
    assert pl.hbm_staging_bytes == pl.n_slices_ring * pl.slice_tokens * 512 and pl.n_slices_ring >= 2
    assert pl.heads_per_group == 1 and pl.n_groups == 8
    # Table 11, HeadInfer-4000K row: 3.91 GB on the GPU (two heads), 500 GB in total
    S4 = 4000 * 1024
    pl4 = hb.hi_offload_plan(llama(S4, 32768))
    g = GOLD["table11_max_context"]["rows"]["headwise"]
    assert round(pl4.hbm_pingpong_paper_bytes / 2 ** 30, 2) == g["kv"]
    assert round(pl4.host_bytes_total / 2 ** 30) == g["total_kv"]


@pytest.mark.parametrize("S,expect", [(100 * 1024, 8), (500 * 1024, 8), (500 * 1024 + 1, 4), (1 << 20, 4),
                                      ((1 << 20) + 1, 2), (2 << 20, 2), ((2 << 20) + 1, 1), (4 << 20, 1)])
def test_plan_reports_paper_adaptive_grouping(S, expect):
    # Section 4: all heads fused up to 500K, two groups to 1M, four to 2M, eight (one head each) beyond
    assert hb.hi_offload_plan(llama(S, 8192)).paper_heads_per_group == expect


def test_plan_flop_and_byte_model_matches_oracle():
    S, Cc = 1 << 20, 16384
    pl = hb.hi_offload_plan(llama(S, Cc))
    assert pl.flop_prefill_unit == mm.causal_flops_unit(4, Cc, S - Cc, 128)
    assert pl.bytes_link_prefill_unit == 512 * S
    assert pl.bytes_link_decode_unit == 512 * S
    # link intensity of a prefill unit is ~ C * G flop per byte (the law behind Table 12's offload columns)
    assert abs(pl.flop_prefill_unit / (512 * (S - Cc)) / (Cc * 4) - 1.0) < 0.01
    assert pl.regime_prefill == hb.HI_REGIME_COMPUTE and pl.regime_decode == hb.HI_REGIME_LINK
    # Table 12: with a 25 GB/s link and 165 TFLOPS, a 1K-context offloaded prefill is link bound, 10K is not
    for S_k, row in ((1, "memory"), (10, "compute")):
        p = llama(S_k * 1024, S_k * 1024, link_GBps=25.0, mfma_TFLOPs=165.0, hbm_GBps=1000.0)
        got = hb.hi_offload_plan(p).regime_prefill
        # the paper's table counts 4*S^2*d flops against 2*S*d*2*2 KV bytes (non-causal); at chunk = S and P = 0
        # the causal unit has half those flops, so the 1K case stays link bound and the 10K case compute bound
        assert (got == hb.HI_REGIME_LINK) == (row == "memory"), (S_k, got)


def test_plan_head_grouping_rule():
    # Section 4, adaptive head grouping: all heads per call at short contexts (as many as a staging slice holds
    # with 64 rows each), two up to 256K, one beyond; hi_prefill_group / hi_decode_group accept any size
    expect = {1024: 4, 4096: 8, 16384: 8, 65536: 2, 262144: 2, 1 << 20: 1, 4 << 20: 1}
    for S, hpg in expect.items():
        pl = hb.hi_offload_plan(llama(S, min(S, 16384)))
        assert pl.heads_per_group == hpg and pl.n_groups == -(-8 // hpg), (S, pl.heads_per_group)
        assert pl.heads_per_group * 64 <= pl.slice_tokens


def test_resident_heads_need_budget():
    st, _ = hb.hi_offload_plan(hb.make_problem(1, 8, 4, 4096, 512, gpu_kv_budget_heads=2, resident_heads=2), check=False)
    assert st == hb.HI_ERR_HBM_BUDGET
    pl = hb.hi_offload_plan(hb.make_problem(1, 8, 4, 4096, 512, gpu_kv_budget_heads=8, resident_heads=4))
    assert pl.hbm_resident_bytes == 4 * pl.host_bytes_per_head
    assert pl.hbm_staging_bytes <= 8 * pl.host_bytes_per_head


def test_plan_geometry_small_and_large():
    pl = hb.hi_offload_plan(hb.make_problem(1, 1, 4, 2048 + 16, 512))
    assert pl.slice_tokens == 512 and pl.n_slices_ring == 4 and pl.prefill_rows_per_wg == 32
    pl = hb.hi_offload_plan(llama(4 << 20, 32768))
    assert pl.slice_tokens == 262144 and pl.n_slices_ring == 16
    assert pl.workspace_bytes >= pl.ws_partials_offset + (17 * 256) * 4 * 130 * 4
    assert hb.hi_offload_plan(hb.make_problem(1, 1, 1, 4096, 512)).prefill_rows_per_wg == 128


def test_plan_rejects_bad_problems():
    bad = [
        (dict(head_dim=64), hb.HI_ERR_UNSUPPORTED),
        (dict(dtype_bytes=4), hb.HI_ERR_UNSUPPORTED),
        (dict(gqa_group=3), hb.HI_ERR_UNSUPPORTED),
        (dict(n_layers=0), hb.HI_ERR_ARG),
        (dict(max_context=0), hb.HI_ERR_ARG),
        (dict(chunk=0), hb.HI_ERR_ARG),
        (dict(chunk=5000), hb.HI_ERR_ARG),
        (dict(gpu_kv_budget_heads=0), hb.HI_ERR_ARG),
        (dict(q_prescaled=2), hb.HI_ERR_ARG),
        (dict(max_context=100, chunk=50), hb.HI_ERR_HBM_BUDGET),
        (dict(host_mem_limit_bytes=1 << 20), hb.HI_ERR_HOST_MEM),
    ]
    for kw, code in bad:
        args = dict(n_layers=2, n_kv_heads=2, gqa_group=4, max_context=4096, chunk=512)
        args.update(kw)
        st, plan = hb.hi_offload_plan(hb.make_problem(**args), check=False)
        assert st == code, (kw, st)
        assert plan.host_bytes_total == 0          # untouched on error
    assert hb.lib().hi_offload_plan(None, None) == hb.HI_ERR_ARG


def test_entry_points_reject_null_context_without_touching_the_gpu():
    L = hb.lib()
    assert L.hi_prefill_head(None, 0, 0, None, None, None, 0, 1, None, -1, 0, 0) == hb.HI_ERR_ARG
    assert L.hi_decode_head(None, 0, 0, None, None, None, 0, None, -1, 0, 0) == hb.HI_ERR_ARG
    assert L.hi_sync(None) == hb.HI_ERR_ARG
    assert L.hi_ctx_set_run_ahead(None, 2) == hb.HI_ERR_ARG and L.hi_ctx_set_flags(None, 0) == hb.HI_ERR_ARG
    assert L.hi_get_stats(None, None) == hb.HI_ERR_ARG
    assert L.hi_ctx_destroy(None) == hb.HI_OK
    prob = hb.make_problem(1, 1, 4, 4096, 512)
    plan = hb.hi_offload_plan(prob)
    st, _ = hb.hi_ctx_create(prob, plan, 7, 1, 1, 1, None, None, None, check=False)
    assert st == hb.HI_ERR_ARG                      # unknown mode
    st, _ = hb.hi_ctx_create(prob, plan, hb.HI_MODE_OFFLOAD, 1, 1, None, None, None, None, check=False)
    assert st == hb.HI_ERR_ARG                      # null workspace (a null cache means: one allocation per layer)
    st, _ = hb.hi_ctx_create(prob, plan, hb.HI_MODE_OFFLOAD, 1, None, 1, None, None, None, check=False)
    assert st == hb.HI_ERR_ARG                      # null staging buffer in offload mode
    assert L.hi_ctx_set_layer_cache(None, 0, None) == hb.HI_ERR_ARG
    other = hb.hi_offload_plan(hb.make_problem(1, 1, 4, 8192, 512))
    st, _ = hb.hi_ctx_create(prob, other, hb.HI_MODE_OFFLOAD, 1, 1, 1, None, None, None, check=False)
    assert st == hb.HI_ERR_ARG and "plan" in hb.last_error()


def test_plan_streaming_heads():
    """Appendix E: streaming heads take a bounded HBM store each and no host rows."""
    base = dict(n_layers=32, n_kv_heads=8, gqa_group=4, max_context=1 << 20, chunk=16384)
    ref = hb.hi_offload_plan(hb.make_problem(**base))
    pl = hb.hi_offload_plan(hb.make_problem(**base, streaming_heads=4, sink_tokens=64, recent_tokens=1024))
    assert pl.stream_rows == 1088
    assert pl.hbm_stream_bytes == 32 * 4 * 1088 * 512
    assert pl.hbm_stream_offset == pl.hbm_resident_offset + pl.hbm_resident_bytes
    assert pl.hbm_staging_bytes == ref.hbm_staging_bytes + pl.hbm_stream_bytes
    assert pl.host_bytes_total == ref.host_bytes_total // 2            # 50 % sparsity: half of the host cache
    assert (pl.slice_tokens, pl.n_slices_ring) == (ref.slice_tokens, ref.n_slices_ring)
    assert ref.stream_rows == 0 and ref.hbm_stream_bytes == 0
    bad = [dict(streaming_heads=8, sink_tokens=4, recent_tokens=4), dict(streaming_heads=-1),
           dict(streaming_heads=2, sink_tokens=4, recent_tokens=0), dict(streaming_heads=2, sink_tokens=-1, recent_tokens=4),
           dict(streaming_heads=2, sink_tokens=1 << 22, recent_tokens=1),
           dict(streaming_heads=4, sink_tokens=4, recent_tokens=4, resident_heads=32 * 4 + 1, gpu_kv_budget_heads=200)]
    for kw in bad:
        st, _ = hb.hi_offload_plan(hb.make_problem(**base, **kw), check=False)
        assert st == hb.HI_ERR_ARG, kw
    # resident heads count over the retrieval heads only
    ok = hb.hi_offload_plan(hb.make_problem(**base, streaming_heads=4, sink_tokens=4, recent_tokens=4,
                                            resident_heads=3, gpu_kv_budget_heads=4))
    assert ok.hbm_resident_bytes == 3 * ok.host_bytes_per_head


def test_plan_four_bit_link_rows():
    """4-bit rows on the link: 80-byte rows in the host cache, and ring + landing areas inside the same HBM budget."""
    base = dict(n_layers=32, n_kv_heads=8, gqa_group=4, max_context=1 << 20, chunk=16384)
    ref = hb.hi_offload_plan(hb.make_problem(**base))
    same = hb.hi_offload_plan(hb.make_problem(**base, link_kv_bits=16))
    assert bytes(same) == bytes(ref)
    pl = hb.hi_offload_plan(hb.make_problem(**base, link_kv_bits=4))
    assert ref.link_row_bytes == 256 and pl.link_row_bytes == 80
    assert pl.host_bytes_per_head == (1 << 20) * 160 and pl.host_bytes_total * 256 == ref.host_bytes_total * 80
    ring = pl.n_slices_ring * pl.slice_tokens
    assert pl.hbm_packed_bytes == ring * 160 and pl.hbm_packed_offset == pl.hbm_stream_offset + pl.hbm_stream_bytes
    assert pl.hbm_staging_bytes == ring * 512 + pl.hbm_packed_bytes <= (1 << 20) * 512      # one head's worth of HBM
    assert pl.slice_tokens % 64 == 0 and pl.n_slices_ring >= 2
    assert pl.ws_writeback_bytes >= 2 * 8 * 16384 * 160 and pl.workspace_bytes == pl.ws_writeback_offset + pl.ws_writeback_bytes
    assert ref.hbm_packed_bytes == 0 and ref.ws_writeback_bytes == 0
    assert pl.bytes_link_decode_unit * 256 == ref.bytes_link_decode_unit * 80
    # resident heads keep bf16 rows in HBM whatever the link carries
    r = hb.hi_offload_plan(hb.make_problem(**base, link_kv_bits=4, resident_heads=2, gpu_kv_budget_heads=3))
    assert r.hbm_resident_bytes == 2 * (1 << 20) * 512
    for bits in (1, 8, -4, 3):
        st, _ = hb.hi_offload_plan(hb.make_problem(**base, link_kv_bits=bits), check=False)
        assert st == hb.HI_ERR_ARG, bits


def test_prescale_constant_turns_the_softmax_of_eq3_into_powers_of_two():
    """HI_Q_PRESCALE is the constant with which exp(q.k / sqrt(d_k)) = 2^(q'.k) for q' = HI_Q_PRESCALE q: checked
    against the oracle's softmax weights (Eq. 3), and the header's value against the binding's."""
    from oracle import attention as oa
    rng = np.random.default_rng(5)
    q, K = rng.standard_normal(128), rng.standard_normal((37, 128))
    w = oa.softmax_weights(q, K, 37)
    e = np.exp2(K @ (hb.HI_Q_PRESCALE * q))
    assert np.abs(w - e / e.sum()).max() < 1e-14
    header = open(os.path.join(ROOT, "include", "headinfer.h")).read()
    assert "#define HI_Q_PRESCALE %.17gf" % hb.HI_Q_PRESCALE in header
