"""Algorithm 1's loops over the per-head entry points, on synthetic inputs (shared by the tests and bench.py).

Loop order is the paper's: chunk -> layer -> head for prefill, token -> layer -> head for decode; every call
names the unit that follows it so the library can prefetch across head, layer, chunk and token boundaries.
Only argument marshalling happens here.
"""
from __future__ import annotations

import torch

from . import synth
from .session import Session


class LayerInputs:
    """Seeded post-RoPE Q/K/V of an attention-only stack, laid out per (chunk, layer, head) unit in HBM:
    q[chunk][layer][kv_head] is [G][C][d], k/v[chunk][layer][kv_head] is [C][d] (the last chunk may be short)."""

    def __init__(self, seed, n_layers, n_kv_heads, G, S, C, device, peaked=False, first_layer=0):
        self.seed, self.L, self.H, self.G, self.S, self.C = seed, n_layers, n_kv_heads, G, S, C
        self.device, self.peaked, self.first_layer = device, peaked, first_layer
        self.q, self.k, self.v = [], [], []
        for p in range(0, S, C):
            n = min(C, S - p)
            ql, kl, vl = [], [], []
            for l in range(n_layers):
                lay = first_layer + l
                ql.append([torch.stack([synth.draw_q(seed, lay, h * G + g, p, n, device=device) for g in range(G)])
                           for h in range(n_kv_heads)])
                kl.append([synth.draw_k(seed, lay, h, p, n, device=device, peaked=peaked) for h in range(n_kv_heads)])
                vl.append([synth.draw_v(seed, lay, h, p, n, device=device) for h in range(n_kv_heads)])
            self.q.append(ql); self.k.append(kl); self.v.append(vl)

    @property
    def n_chunks(self):
        return len(self.q)

    def decode_rows(self, pos):
        """q [L][H][G][d], k, v [L][H][d] of the token at absolute position pos."""
        dev, G = self.device, self.G
        q = [[torch.stack([synth.draw_q(self.seed, self.first_layer + l, h * G + g, pos, 1, device=dev)[0]
                           for g in range(G)]) for h in range(self.H)] for l in range(self.L)]
        k = [[synth.draw_k(self.seed, self.first_layer + l, h, pos, 1, device=dev, peaked=self.peaked)[0]
              for h in range(self.H)] for l in range(self.L)]
        v = [[synth.draw_v(self.seed, self.first_layer + l, h, pos, 1, device=dev)[0] for h in range(self.H)]
             for l in range(self.L)]
        return q, k, v


def _next_unit(L, H, l, h, same_step_past, next_step_past):
    """The unit after (l, h) in layer -> head order, wrapping to the next chunk / token."""
    if h + 1 < H:
        return (l, h + 1, same_step_past)
    if l + 1 < L:
        return (l + 1, 0, same_step_past)
    if next_step_past is None:
        return None
    return (0, 0, next_step_past)


def prefill(ss: Session, inp: LayerInputs, out_buf=None, keep=None, last_hint=None):
    """Chunked head-wise prefill of the whole stack.  out_buf: optional [L][H] list of [G][C][d] tensors that are
    overwritten chunk after chunk; keep(chunk, layer, head, out) is called (on the compute stream) after each unit
    to capture what a test wants to look at.  Returns nothing; call ss.sync() before reading results."""
    L, H, G, C = inp.L, inp.H, inp.G, inp.C
    if out_buf is None:
        out_buf = [[torch.empty(G, C, 128, dtype=ss.out_dtype, device=inp.device) for _ in range(H)] for _ in range(L)]
    for c in range(inp.n_chunks):
        past = c * C
        n = inp.k[c][0][0].shape[0]
        nxt_past = past + n if c + 1 < inp.n_chunks else None
        for l in range(L):
            for h in range(H):
                nxt = _next_unit(L, H, l, h, past, nxt_past)
                if nxt is None:
                    nxt = last_hint
                out = out_buf[l][h][:, :n] if n == C else out_buf[l][h].view(-1)[:G * n * 128].view(G, n, 128)
                ss.prefill_head(l, h, inp.q[c][l][h], inp.k[c][l][h], inp.v[c][l][h], past, out, nxt)
                if keep is not None:
                    keep(c, l, h, out)
    return out_buf


def decode(ss: Session, inp: LayerInputs, start_pos, n_tokens, rows=None, keep=None):
    """n_tokens decode steps at positions start_pos..; rows: optional pre-drawn list of decode_rows() results."""
    L, H, G = inp.L, inp.H, inp.G
    outs = []
    borrowed = []       # rows drawn here: the library borrows them until ss.sync() (the write-back reads k, v)
    for t in range(n_tokens):
        pos = start_pos + t
        q, k, v = rows[t] if rows is not None else inp.decode_rows(pos)
        if rows is None:
            borrowed.append((q, k, v))
        out = torch.empty(L, H, G, 128, dtype=ss.out_dtype, device=inp.device)
        nxt_past = pos + 1 if t + 1 < n_tokens else None
        for l in range(L):
            for h in range(H):
                nxt = _next_unit(L, H, l, h, pos, nxt_past)
                ss.decode_head(l, h, q[l][h], k[l][h], v[l][h], pos, out[l, h], nxt)
        if keep is not None:
            keep(t, out)
        outs.append(out)
    if borrowed:
        # The asynchronous write-backs on the D2H stream still read the drawn rows; freeing them now would hand
        # their blocks back to the allocator of the compute stream.  Keep them until the streams have drained.
        ss.sync()
    return outs
