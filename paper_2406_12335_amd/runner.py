"""Device-buffer bookkeeping for a pruned per-head KV cache.

`PrunedKVCache` owns two sets of cache buffers (compaction is out of place, so the sets
alternate), the workspace and the host-side row counts, and calls the three library entry
points in the order of the method: prompt pass -> prune -> (decode step -> prune)*.
It computes nothing itself.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


class PrunedKVCache:
    def __init__(self, batch: int, n_heads: int, head_dim: int, dtype: torch.dtype, n_sink: int, recent: int,
                 budgets: Sequence[int], device, cap_cache: Optional[int] = None, track_pos: bool = True,
                 ctx=None, norm: int = 0):
        self.device = torch.device(device)
        self.batch, self.n_heads, self.head_dim, self.dtype = batch, n_heads, head_dim, dtype
        self.n_sink, self.recent, self.norm = n_sink, recent, norm
        self.budgets = [int(x) for x in budgets]
        self.cap = int(cap_cache) if cap_cache else max(self.budgets) + 1
        self._own_ctx = ctx is None
        self.ctx = B.vatp_create(self.device.index or 0) if ctx is None else ctx
        shape = (batch, n_heads, self.cap)
        mk = lambda *s, dt: torch.empty(*s, dtype=dt, device=self.device)
        self.K = [mk(*shape, head_dim, dt=dtype) for _ in range(2)]
        self.V = [mk(*shape, head_dim, dt=dtype) for _ in range(2)]
        self.S = [mk(*shape, dt=torch.float32) for _ in range(2)]
        self.nrm = [mk(*shape, dt=torch.float32) for _ in range(2)]
        self.pos = [mk(*shape, dt=torch.int32) for _ in range(2)] if track_pos else [None, None]
        self.kept_idx = mk(*shape, dt=torch.int32)
        self.cur = 0
        self.lens: List[int] = [0] * batch
        self._p_dec = B.Params(batch, n_heads, head_dim, dtype, n_sink, recent, self.cap, self.lens, self.budgets,
                               norm=norm)
        # sized for the fullest cache a decode step may meet (cap - 1 rows plus the new one)
        self._p_dec.set_len([self.cap - 1] * batch)
        nbytes = B.vatp_workspace_bytes(self.ctx, self._p_dec, B.CALL_DECODE_STEP)
        self._p_dec.set_len(self.lens)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        self.S_prompt = self.nrm_prompt = None

    def close(self):
        if self._own_ctx and self.ctx is not None:
            B.vatp_destroy(self.ctx)
            self.ctx = None

    # -- prompt pass -----------------------------------------------------------------
    def prefill_score(self, Q, K, V, lens: Sequence[int], stream=None):
        """vatp_prefill_score on [b, H, cap_p, d] prompt tensors; results kept in S_prompt / nrm_prompt."""
        b, H, cap_p, d = Q.shape
        p = B.Params(b, H, d, self.dtype, self.n_sink, self.recent, cap_p, lens, self.budgets, cap_out=self.cap,
                     norm=self.norm)
        need = B.vatp_workspace_bytes(self.ctx, p, B.CALL_PREFILL_SCORE)
        if getattr(self, "_ws_prompt", None) is None or self._ws_prompt.numel() < need:
            self._ws_prompt = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        if self.S_prompt is None or self.S_prompt.shape != (b, H, cap_p):
            self.S_prompt = torch.empty(b, H, cap_p, dtype=torch.float32, device=self.device)
            self.nrm_prompt = torch.empty(b, H, cap_p, dtype=torch.float32, device=self.device)
        B.vatp_prefill_score(self.ctx, p, Q, K, V, self.S_prompt, self.nrm_prompt, self._ws_prompt, stream)
        self._p_prompt = p
        self._prompt_lens = [int(x) for x in lens]

    def prune_prompt(self, K, V, stream=None):
        """vatp_select_compact from the prompt tensors into cache set 0."""
        p = self._p_prompt
        if self.pos[0] is not None:
            if getattr(self, "_pos_prompt", None) is None or self._pos_prompt.shape != self.S_prompt.shape:
                cap_p = self.S_prompt.shape[-1]
                self._pos_prompt = torch.arange(cap_p, dtype=torch.int32, device=self.device).expand(
                    self.batch, self.n_heads, cap_p).contiguous()
            pos_in = self._pos_prompt
        else:
            pos_in = None
        self.cur = 0
        B.vatp_select_compact(self.ctx, p, K, V, self.S_prompt, self.nrm_prompt, pos_in, self.K[0], self.V[0],
                              self.S[0], self.nrm[0], self.pos[0], self.kept_idx, None, stream)
        self.lens = [min(n, bud) for n, bud in zip(self._prompt_lens, self.budgets)]

    # -- decode ----------------------------------------------------------------------
    def decode_step(self, q, k, v, new_pos: Optional[Sequence[int]], stream=None):
        c = self.cur
        self._p_dec.set_len(self.lens)
        B.vatp_decode_step(self.ctx, self._p_dec, q, k, v, self.K[c], self.V[c], self.S[c], self.nrm[c],
                           self.pos[c], new_pos if self.pos[c] is not None else None, self.ws, stream)
        self.lens = [n + 1 for n in self.lens]

    def prune(self, stream=None):
        c, o = self.cur, 1 - self.cur
        self._p_dec.set_len(self.lens)
        B.vatp_select_compact(self.ctx, self._p_dec, self.K[c], self.V[c], self.S[c], self.nrm[c], self.pos[c],
                              self.K[o], self.V[o], self.S[o], self.nrm[o], self.pos[o], self.kept_idx, None,
                              stream)
        self.cur = o
        self.lens = [min(n, bud) for n, bud in zip(self.lens, self.budgets)]
