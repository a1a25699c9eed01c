"""Buffers, streams and a context for one problem: the thin harness the tests and the benchmark share.

PyTorch is used for device / pinned-host memory and streams only; every step of the path runs in the library.
"""
from __future__ import annotations

import torch

from . import binding as hb


class Session:
    def __init__(self, n_layers, n_kv_heads, gqa_group, max_context, chunk, mode=hb.HI_MODE_OFFLOAD, out_fp32=1,
                 device="cuda:0", gpu_kv_budget_heads=1, n_compute_units=0, resident_heads=0, streaming_heads=0,
                 sink_tokens=0, recent_tokens=0, link_kv_bits=0, per_layer_cache=False, progress=None, streaming_mask=None,
                 q_prescaled=False):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: the library has no CPU path")
        self.device = torch.device(device)
        self.mode = mode
        self.G = gqa_group
        self.problem = hb.make_problem(n_layers, n_kv_heads, gqa_group, max_context, chunk, out_fp32=out_fp32,
                                       gpu_kv_budget_heads=gpu_kv_budget_heads, n_compute_units=n_compute_units,
                                       resident_heads=resident_heads, streaming_heads=streaming_heads,
                                       sink_tokens=sink_tokens, recent_tokens=recent_tokens,
                                       link_kv_bits=link_kv_bits, streaming_mask=streaming_mask,
                                       q_prescaled=int(bool(q_prescaled)))
        # retrieval heads of each layer (the heads that have rows in the cache), in head order
        if streaming_mask is not None:
            self.retrieval = [[h for h in range(n_kv_heads) if not streaming_mask[l][h]] for l in range(n_layers)]
        else:
            self.retrieval = [list(range(n_kv_heads - streaming_heads)) for _ in range(n_layers)]
        self.plan = hb.hi_offload_plan(self.problem)
        nbytes = self.plan.host_bytes_total
        # per_layer_cache: one allocation per layer (hi_ctx_set_layer_cache) instead of one for the whole cache
        self.kv_layers = None
        if per_layer_cache:
            per_head = self.plan.host_bytes_per_head
            per = per_head * len(self.retrieval[0])
            if mode == hb.HI_MODE_OFFLOAD:
                self.kv_layers = []
                for l in range(n_layers):
                    self.kv_layers.append(torch.empty(per_head * len(self.retrieval[l]), dtype=torch.uint8, pin_memory=True))
                    if progress is not None:
                        progress(f"pinned the cache of layer {l + 1} of {n_layers} ({per / 2**30:.1f} GiB)")
            else:
                self.kv_layers = [torch.empty(per_head * len(self.retrieval[l]), dtype=torch.uint8, device=self.device)
                                  for l in range(n_layers)]
            self.kv = None
            nbytes = 0
        if mode == hb.HI_MODE_OFFLOAD:
            if not per_layer_cache:
                self.kv = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
            self.staging = torch.empty(self.plan.hbm_staging_bytes, dtype=torch.uint8, device=self.device)
        else:
            if not per_layer_cache:
                self.kv = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.staging = None
            if self.plan.hbm_stream_bytes > 0:      # only the streaming heads' stores are used
                self.staging = torch.empty(self.plan.hbm_staging_bytes, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(self.plan.workspace_bytes, dtype=torch.uint8, device=self.device)
        self.s_compute = torch.cuda.Stream(self.device)
        self.s_h2d = torch.cuda.Stream(self.device)
        self.s_d2h = torch.cuda.Stream(self.device)
        self.ctx = hb.hi_ctx_create(self.problem, self.plan, mode, self.kv, self.staging, self.workspace,
                                    self.s_compute, self.s_h2d, self.s_d2h)
        if self.kv_layers is not None:
            for l, t in enumerate(self.kv_layers):
                hb.hi_ctx_set_layer_cache(self.ctx, l, t)
        self.out_dtype = torch.float32 if out_fp32 else torch.bfloat16

    # [layer][retrieval kv_head][K|V][S_max][d] bf16 views of the cache (host or device); with 4-bit rows on the
    # link, [layer][retrieval kv_head][K|V][S_max][80] bytes
    def cache_view(self, layer=None) -> torch.Tensor:
        p = self.problem
        if self.kv_layers is not None:          # one allocation per layer: the view of one layer, [1][kv_head]...
            assert layer is not None, "a per-layer cache is viewed layer by layer"
            raw = self.kv_layers[layer]
            if p.link_kv_bits == 4:
                return raw.view(1, p.n_kv_heads - p.streaming_heads, 2, p.max_context, self.plan.link_row_bytes)
            return raw.view(torch.bfloat16).view(1, p.n_kv_heads - p.streaming_heads, 2, p.max_context, p.head_dim)
        if p.link_kv_bits == 4:
            return self.kv.view(p.n_layers, p.n_kv_heads - p.streaming_heads, 2, p.max_context,
                                self.plan.link_row_bytes)
        return self.kv.view(torch.bfloat16).view(p.n_layers, p.n_kv_heads - p.streaming_heads, 2, p.max_context,
                                                 p.head_dim)

    def head_cache_view(self, layer, head) -> torch.Tensor:
        """[K|V][S_max][d] bf16 (or [K|V][S_max][80] bytes) rows of one retrieval head, whatever the head roles."""
        p = self.problem
        j = self.retrieval[layer].index(head)
        per_head = self.plan.host_bytes_per_head
        if self.kv_layers is not None:
            raw = self.kv_layers[layer][j * per_head:(j + 1) * per_head]
        else:
            first = sum(len(self.retrieval[l]) for l in range(layer)) + j
            raw = self.kv[first * per_head:(first + 1) * per_head]
        if p.link_kv_bits == 4:
            return raw.view(2, p.max_context, self.plan.link_row_bytes)
        return raw.view(torch.bfloat16).view(2, p.max_context, p.head_dim)

    # [layer][streaming head][K|V][stream_rows][d] bf16 view of the streaming heads' bounded stores
    def stream_view(self) -> torch.Tensor:
        p, pl = self.problem, self.plan
        raw = self.staging[pl.hbm_stream_offset:pl.hbm_stream_offset + pl.hbm_stream_bytes]
        return raw.view(torch.bfloat16).view(p.n_layers, p.streaming_heads, 2, pl.stream_rows, p.head_dim)

    # [resident head][K|V][S_max][d] bf16 view of the HBM-resident heads' K/V (offload mode, resident_heads > 0)
    def resident_view(self) -> torch.Tensor:
        p, pl = self.problem, self.plan
        raw = self.staging[pl.hbm_resident_offset:pl.hbm_resident_offset + pl.hbm_resident_bytes]
        return raw.view(torch.bfloat16).view(p.resident_heads, 2, p.max_context, p.head_dim)

    def prefill_head(self, layer, head, q, k_new, v_new, past_len, out, nxt=None):
        nl, nh, npast = nxt if nxt is not None else (-1, 0, 0)
        return hb.hi_prefill_head(self.ctx, layer, head, q, k_new, v_new, past_len, k_new.shape[0], out, nl, nh, npast)

    def decode_head(self, layer, head, q, k_new, v_new, past_len, out, nxt=None):
        nl, nh, npast = nxt if nxt is not None else (-1, 0, 0)
        return hb.hi_decode_head(self.ctx, layer, head, q, k_new, v_new, past_len, out, nl, nh, npast)

    def prefill_group(self, layer, head, n_heads, q, k_new, v_new, past_len, out, nxt=None):
        """q [n_heads][G][C][128], k_new / v_new [n_heads][C][128]; nxt = (layer, first head, n_heads, past) or None"""
        nl, nh, nn, npast = nxt if nxt is not None else (-1, 0, 1, 0)
        return hb.hi_prefill_group(self.ctx, layer, head, n_heads, q, k_new, v_new, past_len, k_new.shape[1], out,
                                   nl, nh, nn, npast)

    def decode_group(self, layer, head, n_heads, q, k_new, v_new, past_len, out, nxt=None):
        """q [n_heads][G][128], k_new / v_new [n_heads][128]"""
        nl, nh, nn, npast = nxt if nxt is not None else (-1, 0, 1, 0)
        return hb.hi_decode_group(self.ctx, layer, head, n_heads, q, k_new, v_new, past_len, out, nl, nh, nn, npast)

    def sync(self):
        hb.hi_sync(self.ctx)

    def stats(self):
        return hb.hi_get_stats(self.ctx)

    def close(self):
        if self.ctx is not None:
            hb.hi_sync(self.ctx, check=False)
            hb.hi_ctx_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
