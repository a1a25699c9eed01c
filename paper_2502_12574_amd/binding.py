"""ctypes binding of include/headinfer.h: argument marshalling only, every step runs in the library.

Function names and argument order mirror the C declarations.  Device buffers are passed as torch tensors (their
data_ptr is taken) or raw integer addresses; streams as torch.cuda.Stream objects or raw hipStream_t integers.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libheadinfer.so")

HI_OK, HI_ERR_ARG, HI_ERR_UNSUPPORTED, HI_ERR_HBM_BUDGET = 0, -1, -2, -3
HI_ERR_HOST_MEM, HI_ERR_RANGE, HI_ERR_NOT_PINNED, HI_ERR_HIP = -4, -5, -6, -7
HI_MODE_OFFLOAD, HI_MODE_RESIDENT = 0, 1
HI_REGIME_COMPUTE, HI_REGIME_LINK, HI_REGIME_HBM = 0, 1, 2
HI_FLAG_SKIP_KERNELS, HI_FLAG_SKIP_COPIES, HI_FLAG_TIME_KERNELS = 1, 2, 4
HI_FLAG_PREFILL_NARROW, HI_FLAG_PREFILL_PAIRED, HI_FLAG_PREFILL_DEEP, HI_FLAG_PREFILL_UNPAIRED = 8, 16, 32, 64
HI_FLAG_INJECT_FAILURE = 128
HI_FLAG_PREFILL_MFMA32 = 256
HI_FLAG_PREFILL_8WAVE, HI_FLAG_PREFILL_WIDE, HI_FLAG_PREFILL_SINGLE_SLICES = 512, 1024, 2048
HI_Q_PRESCALE = 0.12751743082459868      # log2(e) / sqrt(128): a pre-scaled query is this times the q of Eq. 3

EXPORTS = ("hi_offload_plan", "hi_ctx_create", "hi_ctx_destroy", "hi_ctx_set_layer_cache", "hi_ctx_set_flags", "hi_ctx_set_run_ahead",
           "hi_prefill_head", "hi_decode_head", "hi_prefill_group", "hi_decode_group", "hi_decode_group_ragged", "hi_proj_workspace_bytes",
           "hi_qkv_rope", "hi_qkv_rope_static", "hi_out_proj", "hi_kv_quantize", "hi_kv_dequantize", "hi_sync", "hi_get_stats", "hi_reset_stats", "hi_status_string", "hi_last_error")


class hi_problem(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("gqa_group", C.c_int32),
                ("head_dim", C.c_int32), ("max_context", C.c_int64), ("chunk", C.c_int32),
                ("gpu_kv_budget_heads", C.c_int32), ("dtype_bytes", C.c_int32), ("out_fp32", C.c_int32),
                ("n_compute_units", C.c_int32), ("resident_heads", C.c_int32), ("host_mem_limit_bytes", C.c_int64),
                ("link_GBps", C.c_double), ("hbm_GBps", C.c_double), ("mfma_TFLOPs", C.c_double),
                ("streaming_heads", C.c_int32), ("sink_tokens", C.c_int32), ("recent_tokens", C.c_int32),
                ("link_kv_bits", C.c_int32), ("streaming_mask", C.c_void_p), ("q_prescaled", C.c_int32)]


class hi_plan(C.Structure):
    _fields_ = [("heads_per_group", C.c_int32), ("n_groups", C.c_int32), ("paper_heads_per_group", C.c_int32),
                ("n_slices_ring", C.c_int32), ("slice_tokens", C.c_int64), ("n_split_decode", C.c_int32),
                ("prefill_rows_per_wg", C.c_int32), ("host_bytes_per_head", C.c_int64),
                ("host_bytes_total", C.c_int64), ("hbm_staging_bytes", C.c_int64),
                ("hbm_pingpong_paper_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("ws_partials_offset", C.c_int64), ("alpha", C.c_double), ("flop_prefill_unit", C.c_double),
                ("bytes_link_prefill_unit", C.c_double), ("bytes_link_decode_unit", C.c_double),
                ("t_comp_prefill_s", C.c_double), ("t_link_prefill_s", C.c_double), ("t_hbm_prefill_s", C.c_double),
                ("t_comp_decode_s", C.c_double), ("t_link_decode_s", C.c_double), ("t_hbm_decode_s", C.c_double),
                ("regime_prefill", C.c_int32), ("regime_decode", C.c_int32),
                ("hbm_resident_offset", C.c_int64), ("hbm_resident_bytes", C.c_int64),
                ("hbm_stream_offset", C.c_int64), ("hbm_stream_bytes", C.c_int64), ("stream_rows", C.c_int64),
                ("link_row_bytes", C.c_int64), ("hbm_packed_offset", C.c_int64), ("hbm_packed_bytes", C.c_int64),
                ("ws_writeback_offset", C.c_int64), ("ws_writeback_bytes", C.c_int64)]


class hi_stats(C.Structure):
    _fields_ = [("bytes_h2d", C.c_int64), ("bytes_d2h", C.c_int64), ("n_h2d_copies", C.c_int64),
                ("n_d2h_copies", C.c_int64), ("n_prefill_kernels", C.c_int64), ("n_decode_kernels", C.c_int64),
                ("n_combine_kernels", C.c_int64), ("peak_staging_bytes", C.c_int64),
                ("prefill_kernel_ms", C.c_double), ("decode_kernel_ms", C.c_double),
                ("h2d_copy_ms", C.c_double), ("d2h_copy_ms", C.c_double), ("exposed_copy_ms", C.c_double)]


class HiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({last_error()})")


_lib = None


def lib() -> C.CDLL:
    """Load libheadinfer.so (built by paper_2502_12574_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2502_12574_amd.build` first; "
                               "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.hi_offload_plan.argtypes = [C.POINTER(hi_problem), C.POINTER(hi_plan)]
        L.hi_ctx_create.argtypes = [C.POINTER(hi_problem), C.POINTER(hi_plan), i32, vp, vp, vp, vp, vp, vp,
                                    C.POINTER(vp)]
        L.hi_ctx_destroy.argtypes = [vp]
        L.hi_ctx_set_layer_cache.argtypes = [vp, i32, vp]
        L.hi_ctx_set_flags.argtypes = [vp, i32]
        L.hi_ctx_set_run_ahead.argtypes = [vp, i32]
        L.hi_prefill_head.argtypes = [vp, i32, i32, vp, vp, vp, i64, i32, vp, i32, i32, i64]
        L.hi_decode_head.argtypes = [vp, i32, i32, vp, vp, vp, i64, vp, i32, i32, i64]
        L.hi_prefill_group.argtypes = [vp, i32, i32, i32, vp, vp, vp, i64, i32, vp, i32, i32, i32, i64]
        L.hi_decode_group.argtypes = [vp, i32, i32, i32, vp, vp, vp, i64, vp, i32, i32, i32, i64]
        L.hi_decode_group_ragged.argtypes = [vp, i32, i32, i32, vp, vp, vp, C.POINTER(i64), vp]
        L.hi_proj_workspace_bytes.argtypes = [i32, C.POINTER(i64)]
        L.hi_qkv_rope.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, C.c_double, i32, vp, vp, vp, vp, C.c_float]
        L.hi_qkv_rope_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, C.c_double, i32, vp, vp, vp, C.c_float]
        L.hi_out_proj.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
        L.hi_kv_quantize.argtypes = [vp, vp, i64, vp]
        L.hi_kv_dequantize.argtypes = [vp, vp, i64, vp]
        L.hi_sync.argtypes = [vp]
        L.hi_get_stats.argtypes = [vp, C.POINTER(hi_stats)]
        L.hi_reset_stats.argtypes = [vp]
        L.hi_status_string.argtypes = [i32]
        for name in EXPORTS:
            getattr(L, name).restype = i32
        L.hi_status_string.restype = C.c_char_p
        L.hi_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hi_status_string(status).decode()


def last_error() -> str:
    return lib().hi_last_error().decode()


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def make_problem(n_layers, n_kv_heads, gqa_group, max_context, chunk, head_dim=128, gpu_kv_budget_heads=1,
                 dtype_bytes=2, out_fp32=0, n_compute_units=0, host_mem_limit_bytes=0, link_GBps=0.0, hbm_GBps=0.0,
                 mfma_TFLOPs=0.0, resident_heads=0, streaming_heads=0, sink_tokens=0, recent_tokens=0,
                 link_kv_bits=0, streaming_mask=None, q_prescaled=0) -> hi_problem:
    """streaming_mask: optional [n_layers][n_kv_heads] nested list / array of 0 and 1 (1 = streaming head).
    q_prescaled: 1 = the queries handed to the attention calls already carry HI_Q_PRESCALE."""
    p = hi_problem(n_layers, n_kv_heads, gqa_group, head_dim, max_context, chunk, gpu_kv_budget_heads,
                   dtype_bytes, out_fp32, n_compute_units, resident_heads, host_mem_limit_bytes, link_GBps, hbm_GBps,
                   mfma_TFLOPs, streaming_heads, sink_tokens, recent_tokens, link_kv_bits, None, int(q_prescaled))
    if streaming_mask is not None:
        flat = [int(x) for row in streaming_mask for x in row]
        assert len(flat) == n_layers * n_kv_heads
        buf = (C.c_uint8 * len(flat))(*flat)
        p._mask_keepalive = buf                       # the struct only holds the address
        p.streaming_mask = C.addressof(buf)
    return p


def hi_offload_plan(problem: hi_problem, check: bool = True):
    plan = hi_plan()
    st = lib().hi_offload_plan(C.byref(problem), C.byref(plan))
    if check and st != HI_OK:
        raise HiError(st, "hi_offload_plan")
    return plan if check else (st, plan)


def hi_ctx_create(problem, plan, mode, kv_cache, hbm_staging, hbm_workspace, stream_compute, stream_h2d,
                  stream_d2h, check: bool = True):
    ctx = C.c_void_p()
    st = lib().hi_ctx_create(C.byref(problem), C.byref(plan), mode, _ptr(kv_cache), _ptr(hbm_staging),
                             _ptr(hbm_workspace), _stream(stream_compute), _stream(stream_h2d),
                             _stream(stream_d2h), C.byref(ctx))
    if check and st != HI_OK:
        raise HiError(st, "hi_ctx_create")
    return ctx if check else (st, ctx)


def hi_ctx_destroy(ctx):
    return lib().hi_ctx_destroy(ctx)


def hi_ctx_set_layer_cache(ctx, layer: int, kv_layer, check: bool = True):
    st = lib().hi_ctx_set_layer_cache(ctx, layer, _ptr(kv_layer))
    if check and st != HI_OK:
        raise HiError(st, "hi_ctx_set_layer_cache")
    return st


def hi_ctx_set_flags(ctx, flags: int, check: bool = True):
    st = lib().hi_ctx_set_flags(ctx, flags)
    if check and st != HI_OK:
        raise HiError(st, "hi_ctx_set_flags")
    return st


def hi_ctx_set_run_ahead(ctx, units: int, check: bool = True):
    st = lib().hi_ctx_set_run_ahead(ctx, units)
    if check and st != HI_OK:
        raise HiError(st, "hi_ctx_set_run_ahead")
    return st


def hi_prefill_head(ctx, layer, kv_head, q_dev, k_new_dev, v_new_dev, past_len, chunk_len, out_dev,
                    next_layer=-1, next_kv_head=0, next_past_len=0, check: bool = True):
    st = lib().hi_prefill_head(ctx, layer, kv_head, _ptr(q_dev), _ptr(k_new_dev), _ptr(v_new_dev), past_len,
                               chunk_len, _ptr(out_dev), next_layer, next_kv_head, next_past_len)
    if check and st != HI_OK:
        raise HiError(st, "hi_prefill_head")
    return st


def hi_decode_head(ctx, layer, kv_head, q_dev, k_new_dev, v_new_dev, past_len, out_dev, next_layer=-1,
                   next_kv_head=0, next_past_len=0, check: bool = True):
    st = lib().hi_decode_head(ctx, layer, kv_head, _ptr(q_dev), _ptr(k_new_dev), _ptr(v_new_dev), past_len,
                              _ptr(out_dev), next_layer, next_kv_head, next_past_len)
    if check and st != HI_OK:
        raise HiError(st, "hi_decode_head")
    return st


def hi_prefill_group(ctx, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, chunk_len, out_dev,
                     next_layer=-1, next_kv_head=0, next_n_heads=1, next_past_len=0, check: bool = True):
    st = lib().hi_prefill_group(ctx, layer, kv_head, n_heads, _ptr(q_dev), _ptr(k_new_dev), _ptr(v_new_dev), past_len,
                                chunk_len, _ptr(out_dev), next_layer, next_kv_head, next_n_heads, next_past_len)
    if check and st != HI_OK:
        raise HiError(st, "hi_prefill_group")
    return st


def hi_decode_group(ctx, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, out_dev, next_layer=-1,
                    next_kv_head=0, next_n_heads=1, next_past_len=0, check: bool = True):
    st = lib().hi_decode_group(ctx, layer, kv_head, n_heads, _ptr(q_dev), _ptr(k_new_dev), _ptr(v_new_dev), past_len,
                               _ptr(out_dev), next_layer, next_kv_head, next_n_heads, next_past_len)
    if check and st != HI_OK:
        raise HiError(st, "hi_decode_group")
    return st


def hi_decode_group_ragged(ctx, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_lens, out_dev,
                           check: bool = True):
    lens = (C.c_int64 * n_heads)(*[int(x) for x in past_lens])
    st = lib().hi_decode_group_ragged(ctx, layer, kv_head, n_heads, _ptr(q_dev), _ptr(k_new_dev), _ptr(v_new_dev), lens,
                                      _ptr(out_dev))
    if check and st != HI_OK:
        raise HiError(st, "hi_decode_group_ragged")
    return st


def hi_proj_workspace_bytes(chunk_len: int) -> int:
    n = C.c_int64()
    st = lib().hi_proj_workspace_bytes(chunk_len, C.byref(n))
    if st != HI_OK:
        raise HiError(st, "hi_proj_workspace_bytes")
    return n.value


def hi_qkv_rope(stream, x_dev, w_qkv_dev, d_model, n_q_heads, n_kv_heads, chunk_len, past_len, rope_theta, out_fp32,
                q_out_dev, k_out_dev, v_out_dev, workspace_dev, q_scale: float = 1.0, check: bool = True):
    st = lib().hi_qkv_rope(_stream(stream), _ptr(x_dev), _ptr(w_qkv_dev), d_model, n_q_heads, n_kv_heads, chunk_len,
                           past_len, float(rope_theta), out_fp32, _ptr(q_out_dev), _ptr(k_out_dev), _ptr(v_out_dev),
                           _ptr(workspace_dev), float(q_scale))
    if check and st != HI_OK:
        raise HiError(st, "hi_qkv_rope")
    return st


def hi_qkv_rope_static(stream, x_dev, w_qkv_dev, d_model, n_q_heads, n_kv_heads, chunk_len, past_len, rope_theta,
                       out_fp32, q_out_dev, k_out_dev, v_out_dev, q_scale: float = 1.0, check: bool = True):
    st = lib().hi_qkv_rope_static(_stream(stream), _ptr(x_dev), _ptr(w_qkv_dev), d_model, n_q_heads, n_kv_heads,
                                  chunk_len, past_len, float(rope_theta), out_fp32, _ptr(q_out_dev), _ptr(k_out_dev),
                                  _ptr(v_out_dev), float(q_scale))
    if check and st != HI_OK:
        raise HiError(st, "hi_qkv_rope_static")
    return st


def hi_out_proj(stream, attn_dev, w_o_dev, n_q_heads, d_model, chunk_len, out_fp32, y_out_dev, check: bool = True):
    st = lib().hi_out_proj(_stream(stream), _ptr(attn_dev), _ptr(w_o_dev), n_q_heads, d_model, chunk_len, out_fp32,
                           _ptr(y_out_dev))
    if check and st != HI_OK:
        raise HiError(st, "hi_out_proj")
    return st


def hi_kv_quantize(stream, rows_dev, n_rows, packed_dev, check: bool = True):
    st = lib().hi_kv_quantize(_stream(stream), _ptr(rows_dev), n_rows, _ptr(packed_dev))
    if check and st != HI_OK:
        raise HiError(st, "hi_kv_quantize")
    return st


def hi_kv_dequantize(stream, packed_dev, n_rows, rows_dev, check: bool = True):
    st = lib().hi_kv_dequantize(_stream(stream), _ptr(packed_dev), n_rows, _ptr(rows_dev))
    if check and st != HI_OK:
        raise HiError(st, "hi_kv_dequantize")
    return st


def hi_sync(ctx, check: bool = True):
    st = lib().hi_sync(ctx)
    if check and st != HI_OK:
        raise HiError(st, "hi_sync")
    return st


def hi_get_stats(ctx) -> hi_stats:
    s = hi_stats()
    st = lib().hi_get_stats(ctx, C.byref(s))
    if st != HI_OK:
        raise HiError(st, "hi_get_stats")
    return s


def hi_reset_stats(ctx):
    st = lib().hi_reset_stats(ctx)
    if st != HI_OK:
        raise HiError(st, "hi_reset_stats")
    return st
