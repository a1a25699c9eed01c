"""Algorithm 1's loops over the per-head entry points, on synthetic inputs (shared by the tests and bench.py).

Loop order is the paper's: chunk -> layer -> head for prefill, token -> layer -> head for decode; every call
names the unit that follows it so the library can prefetch across head, layer, chunk and token boundaries.
With heads_per_call > 1 the head loop advances by groups of consecutive KV heads (Section 4, adaptive head-wise
offloading).  Only argument marshalling happens here.
"""
from __future__ import annotations

import torch

from . import synth
from .session import Session


class LayerInputs:
    """Seeded post-RoPE Q/K/V of an attention-only stack, laid out per (chunk, layer) in HBM with the KV heads of a
    layer stacked: q[chunk][layer] is [H][G][C][d], k/v[chunk][layer] is [H][C][d] (the last chunk may be short), so
    q[chunk][layer][kv_head] is the [G][C][d] operand of a one-head call and a slice of heads that of a group call."""

    def __init__(self, seed, n_layers, n_kv_heads, G, S, C, device, peaked=False, first_layer=0, q_scale=1.0):
        """q_scale: constant folded into the queries (binding.HI_Q_PRESCALE for a Session with q_prescaled)."""
        self.seed, self.L, self.H, self.G, self.S, self.C = seed, n_layers, n_kv_heads, G, S, C
        self.device, self.peaked, self.first_layer, self.q_scale = device, peaked, first_layer, q_scale
        self.q, self.k, self.v = [], [], []
        for p in range(0, S, C):
            n = min(C, S - p)
            ql, kl, vl = [], [], []
            for l in range(n_layers):
                lay = first_layer + l
                ql.append(torch.stack([torch.stack([synth.draw_q(seed, lay, h * G + g, p, n, device=device, scale=q_scale)
                                                    for g in range(G)]) for h in range(n_kv_heads)]))
                kl.append(torch.stack([synth.draw_k(seed, lay, h, p, n, device=device, peaked=peaked)
                                       for h in range(n_kv_heads)]))
                vl.append(torch.stack([synth.draw_v(seed, lay, h, p, n, device=device) for h in range(n_kv_heads)]))
            self.q.append(ql); self.k.append(kl); self.v.append(vl)

    @property
    def n_chunks(self):
        return len(self.q)

    def single_layer(self, l):
        """The same tensors seen as a one-layer stack (layer l), for a run over one layer of the inputs."""
        one = object.__new__(LayerInputs)
        one.__dict__.update(self.__dict__)
        one.L, one.first_layer = 1, self.first_layer + l
        one.q = [[c[l]] for c in self.q]
        one.k = [[c[l]] for c in self.k]
        one.v = [[c[l]] for c in self.v]
        return one

    def decode_rows(self, pos):
        """q [L][H][G][d], k, v [L][H][d] of the token at absolute position pos (lists over layers of stacked heads)."""
        dev, G = self.device, self.G
        q = [torch.stack([torch.stack([synth.draw_q(self.seed, self.first_layer + l, h * G + g, pos, 1, device=dev,
                                                    scale=self.q_scale)[0]
                                       for g in range(G)]) for h in range(self.H)]) for l in range(self.L)]
        k = [torch.stack([synth.draw_k(self.seed, self.first_layer + l, h, pos, 1, device=dev, peaked=self.peaked)[0]
                          for h in range(self.H)]) for l in range(self.L)]
        v = [torch.stack([synth.draw_v(self.seed, self.first_layer + l, h, pos, 1, device=dev)[0] for h in range(self.H)])
             for l in range(self.L)]
        return q, k, v


def _next_unit(L, H, hpc, l, h, same_step_past, next_step_past):
    """The unit after the group starting at (l, h) in layer -> head order, wrapping to the next chunk / token:
    (layer, first head, heads, past) or None."""
    if h + hpc < H:
        return (l, h + hpc, min(hpc, H - h - hpc), same_step_past)
    if l + 1 < L:
        return (l + 1, 0, min(hpc, H), same_step_past)
    if next_step_past is None:
        return None
    return (0, 0, min(hpc, H), next_step_past)


def prefill(ss: Session, inp: LayerInputs, out_buf=None, keep=None, last_hint=None, heads_per_call=1):
    """Chunked head-wise prefill of the whole stack.  out_buf: optional [L] list of [H][G][C][d] tensors that are
    overwritten chunk after chunk; keep(chunk, layer, head, out) is called (on the compute stream) after each unit,
    once per head, to capture what a test wants to look at; last_hint: (layer, head, past) of the unit that follows
    the last one.  Returns out_buf; call ss.sync() before reading results."""
    L, H, G, C, hpc = inp.L, inp.H, inp.G, inp.C, heads_per_call
    if out_buf is None:
        out_buf = [torch.empty(H, G, C, 128, dtype=ss.out_dtype, device=inp.device) for _ in range(L)]
    if last_hint is not None and len(last_hint) == 3:
        last_hint = (last_hint[0], last_hint[1], min(hpc, H), last_hint[2])
    for c in range(inp.n_chunks):
        past = c * C
        n = inp.k[c][0].shape[1]
        nxt_past = past + n if c + 1 < inp.n_chunks else None
        for l in range(L):
            for h in range(0, H, hpc):
                nh = min(hpc, H - h)
                nxt = _next_unit(L, H, hpc, l, h, past, nxt_past)
                if nxt is None:
                    nxt = last_hint
                ob = out_buf[l][h:h + nh]
                out = ob[:, :, :n] if n == C else ob.reshape(-1)[:nh * G * n * 128].view(nh, G, n, 128)
                if hpc == 1:
                    ss.prefill_head(l, h, inp.q[c][l][h], inp.k[c][l][h], inp.v[c][l][h], past, out[0],
                                    None if nxt is None else (nxt[0], nxt[1], nxt[3]))
                else:
                    ss.prefill_group(l, h, nh, inp.q[c][l][h:h + nh], inp.k[c][l][h:h + nh], inp.v[c][l][h:h + nh], past,
                                     out, nxt)
                if keep is not None:
                    for j in range(nh):
                        keep(c, l, h + j, out[j])
    return out_buf


def decode(ss: Session, inp: LayerInputs, start_pos, n_tokens, rows=None, keep=None, heads_per_call=1):
    """n_tokens decode steps at positions start_pos..; rows: optional pre-drawn list of decode_rows() results.
    Returns the outputs, one [L][H][G][d] tensor per token."""
    L, H, G, hpc = inp.L, inp.H, inp.G, heads_per_call
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
            for h in range(0, H, hpc):
                nh = min(hpc, H - h)
                nxt = _next_unit(L, H, hpc, l, h, pos, nxt_past)
                if hpc == 1:
                    ss.decode_head(l, h, q[l][h], k[l][h], v[l][h], pos, out[l, h],
                                   None if nxt is None else (nxt[0], nxt[1], nxt[3]))
                else:
                    ss.decode_group(l, h, nh, q[l][h:h + nh], k[l][h:h + nh], v[l][h:h + nh], pos, out[l, h:h + nh], nxt)
        if keep is not None:
            keep(t, out)
        outs.append(out)
    if borrowed:
        # The asynchronous write-backs on the D2H stream still read the drawn rows; freeing them now would hand
        # their blocks back to the allocator of the compute stream.  Keep them until the streams have drained.
        ss.sync()
    return outs
