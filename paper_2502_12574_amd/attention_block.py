"""One layer's attention block on top of the library: hidden states -> Q/K/V projection with rotary embedding
(hi_qkv_rope) -> head-wise attention with offloaded / resident / streaming KV heads (hi_prefill_group,
hi_decode_group, Algorithm 1's head loop) -> output projection (hi_out_proj).

Only buffers and call order live here; every step runs in the library.  The projection writes Q, K and V
head-major, which is what the attention calls read, and the attention calls write the head-major block the
output projection reads: nothing is reshuffled in between.
"""
from __future__ import annotations

import torch

from . import binding as hb
from .session import Session


class AttentionBlock:
    """The attention block of layer `layer` of a Session (the Session owns the K/V cache of all layers).

    w_qkv [(Hq + 2 Hkv) * 128][d_model] (rows of W_Q, W_K, W_V) and w_o [d_model][Hq * 128], bf16 on the device.
    Heads are called in groups of plan.heads_per_group, retrieval heads first, then the streaming heads."""

    def __init__(self, ss: Session, layer: int, w_qkv: torch.Tensor, w_o: torch.Tensor, rope_theta: float = 500000.0):
        p = ss.problem
        self.ss, self.layer, self.theta = ss, layer, rope_theta
        self.Hkv, self.G, self.Hq, self.D = p.n_kv_heads, p.gqa_group, p.n_kv_heads * p.gqa_group, w_o.shape[0]
        assert w_qkv.shape == ((self.Hq + 2 * self.Hkv) * 128, self.D) and w_o.shape == (self.D, self.Hq * 128)
        self.w_qkv, self.w_o = w_qkv, w_o
        C, dev = p.chunk, ss.device
        self.q = torch.empty(self.Hq * C * 128, dtype=torch.bfloat16, device=dev)
        # K/V of a call are borrowed by its asynchronous write-back to the host: two sets, used in turn, and a set
        # is written again only after the write-back stream has passed the call that last used it
        self.kv = [(torch.empty(self.Hkv * C * 128, dtype=torch.bfloat16, device=dev),
                    torch.empty(self.Hkv * C * 128, dtype=torch.bfloat16, device=dev)) for _ in range(2)]
        self.kv_done = [None, None]
        self.turn = 0
        self.attn = torch.empty(self.Hq * C * 128, dtype=torch.bfloat16, device=dev)
        self.ws = torch.empty(hb.hi_proj_workspace_bytes(C), dtype=torch.uint8, device=dev)
        n_ret, g = self.Hkv - p.streaming_heads, max(1, ss.plan.heads_per_group)
        self.calls = [(h, min(g, n_ret - h)) for h in range(0, n_ret, g)]
        self.calls += [(h, min(g, self.Hkv - h)) for h in range(n_ret, self.Hkv, g)]

    def _views(self, n):
        q = self.q[:self.Hq * n * 128].view(self.Hkv, self.G, n, 128)
        k = self.kv[self.turn][0][:self.Hkv * n * 128].view(self.Hkv, n, 128)
        v = self.kv[self.turn][1][:self.Hkv * n * 128].view(self.Hkv, n, 128)
        o = self.attn[:self.Hq * n * 128].view(self.Hkv, self.G, n, 128)
        return q, k, v, o

    def forward(self, x: torch.Tensor, past_len: int, y: torch.Tensor, nxt=None):
        """x [n][d_model] bf16 hidden states of the tokens at positions past_len .., n = 1 for a decode step;
        y [n][d_model] bf16 receives the block's output.  nxt: the (layer, first head, heads, past) unit that will
        be called after this block's last one, for the prefetch.  Enqueues on the Session's compute stream."""
        ss, n = self.ss, x.shape[0]
        assert ss.out_dtype == torch.bfloat16, "the output projection reads bf16 attention outputs"
        q, k, v, o = self._views(n)
        s = ss.s_compute
        if self.kv_done[self.turn] is not None:
            s.wait_event(self.kv_done[self.turn])
        with torch.cuda.stream(s):
            # the softmax scale rides on the queries when the Session's attention calls expect it there
            hb.hi_qkv_rope(s, x, self.w_qkv, self.D, self.Hq, self.Hkv, n, past_len, self.theta, 0, q, k, v, self.ws,
                           q_scale=hb.HI_Q_PRESCALE if ss.problem.q_prescaled else 1.0)
            for i, (h0, nh) in enumerate(self.calls):
                hint = (self.layer, self.calls[i + 1][0], self.calls[i + 1][1], past_len) if i + 1 < len(self.calls) else nxt
                if n == 1:
                    ss.decode_group(self.layer, h0, nh, q[h0:h0 + nh, :, 0], k[h0:h0 + nh, 0], v[h0:h0 + nh, 0], past_len,
                                    o[h0:h0 + nh, :, 0], hint)
                else:
                    ss.prefill_group(self.layer, h0, nh, q[h0:h0 + nh], k[h0:h0 + nh], v[h0:h0 + nh], past_len,
                                     o[h0:h0 + nh], hint)
            hb.hi_out_proj(s, o, self.w_o, self.Hq, self.D, n, 0, y)
        ev = torch.cuda.Event()
        ev.record(ss.s_d2h)
        self.kv_done[self.turn] = ev
        self.turn ^= 1
        return y
