"""Control flow of the paper's inference pipeline (Algorithm 1) for ONE layer's KV cache, on top of
the C-ABI calls: ckv_schedule_annealed + ckv_compress after prefill, then per decode step
ckv_append, ckv_decode_attn and, once the cache holds budget + g tokens, one clustering round
(ckv_compress with the cache's degrees).  This class holds buffers and decides WHEN to call; every
arithmetic step runs in the library's kernels.  All sequences of the batch share one length."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import (append, budget_tokens, compress, decode_attn, decode_attn_workspace, layout_of, make_params, plan,
               schedule_annealed)


class OnlineCache:
    def __init__(self, K: torch.Tensor, V: torch.Tensor, chunk: int, cache_ratio: float, g: int,
                 q_heads: int, r_init: float = 0.8, delta_r: float = 0.2, r_floor: float = 0.2,
                 n_sink: int = 16, n_recent: int = 64, r_decode: Optional[Sequence[float]] = None):
        """K, V: the prompt's cache [batch, heads, n, dim] after prefill.  Budget B = floor(R*n)
        (Algorithm 1).  The first clustering runs the annealed schedule (Eq. 4, with a floor so the
        loop ends) until the cache fits the budget.  `r_decode`: merge fraction of the k-th
        decode-time round (the last entry repeats); default: r_init every time (the round index of
        Eq. 4 restarts with each clustering episode)."""
        B, H, n, D = K.shape
        self.chunk, self.g, self.n_sink, self.n_recent = chunk, g, n_sink, n_recent
        self.budget = budget_tokens(cache_ratio, n)
        self.r_decode = list(r_decode) if r_decode else [r_init]
        self.capacity = max(self.budget + g, 1)
        self.rounds_prefill = schedule_annealed(n, chunk, self.budget, r_init, delta_r, r_floor, n_sink, n_recent)
        mk = lambda: (torch.empty((B, H, self.capacity, D), dtype=K.dtype, device=K.device),
                      torch.empty((B, H, self.capacity, D), dtype=K.dtype, device=K.device),
                      torch.empty((B, H, self.capacity), dtype=torch.int32, device=K.device))
        self.bufs = [mk(), mk()]
        self.cur = 0
        self.n_clusterings = 0
        # workspaces sized once for the largest calls (a full cache; one round)
        full = self.bufs[0][0]
        one_round = make_params(chunk, rounds=[1.0], n_sink=n_sink, n_recent=n_recent)
        self.ws_round = torch.empty(max(plan(layout_of(full), one_round).workspace_bytes, 256), dtype=torch.uint8,
                                    device=K.device)
        self.ws_attn = torch.zeros(decode_attn_workspace(layout_of(full), q_heads), dtype=torch.uint8,
                                   device=K.device)
        cK, cV, cdeg = self.bufs[0]
        if self.rounds_prefill:
            pl = plan(layout_of(K), make_params(chunk, rounds=self.rounds_prefill, n_sink=n_sink, n_recent=n_recent))
            self.s = pl.out_seq
            compress(K, V, chunk, rounds=self.rounds_prefill, want_assign=False, out=(cK, cV, cdeg, None),
                     n_sink=n_sink, n_recent=n_recent)
        else:                                   # already within budget: zero rounds copy the cache over
            self.s = n
            compress(K, V, chunk, retain_ratio=1.0, want_assign=False, out=(cK, cV, cdeg, None))

    def view(self):
        """(K, V, deg) of the current cache, [batch, heads, s, ...] views of the buffers."""
        cK, cV, cdeg = self.bufs[self.cur]
        return cK[:, :, :self.s], cV[:, :, :self.s], cdeg[:, :, :self.s]

    def step(self, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, out_dtype=None) -> torch.Tensor:
        """One decode step of Algorithm 1; returns the attention output [batch, q_heads, dim]."""
        cK, cV, cdeg = self.bufs[self.cur]
        append(k_new, v_new, cK, cV, cdeg, pos=self.s)
        self.s += 1
        K, V, deg = self.view()
        o = decode_attn(q, K, V, deg=deg, out_dtype=out_dtype, workspace=self.ws_attn)
        if self.s >= self.budget + self.g:
            r = self.r_decode[min(self.n_clusterings, len(self.r_decode) - 1)]
            nxt = self.bufs[1 - self.cur]
            pl = plan(layout_of(K), make_params(self.chunk, rounds=[r], n_sink=self.n_sink, n_recent=self.n_recent))
            compress(K, V, self.chunk, rounds=[r], deg=deg, want_assign=False, out=(nxt[0], nxt[1], nxt[2], None),
                     workspace=self.ws_round, n_sink=self.n_sink, n_recent=self.n_recent)
            self.cur, self.s = 1 - self.cur, pl.out_seq
            self.n_clusterings += 1
        return o
