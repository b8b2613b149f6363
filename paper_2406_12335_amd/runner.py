"""Device-buffer bookkeeping for a pruned per-head KV cache.

`PrunedKVCache` owns two sets of cache buffers (compaction is out of place, so the sets
alternate), the workspace and the host-side row counts, and calls the three library entry
points in the order of the method: prompt pass -> prune -> (decode step -> prune)*.
It computes nothing itself.
"""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence

import torch

from . import binding as B


class PrunedKVCache:
    def __init__(self, batch: int, n_heads: int, head_dim: int, dtype: torch.dtype, n_sink: int, recent: int,
                 budgets: Sequence[int], device, cap_cache: Optional[int] = None, track_pos: bool = True,
                 ctx=None, norm: int = 0, window: Optional[int] = None, q_per_kv: int = 1):
        self.device = torch.device(device)
        self.batch, self.n_heads, self.head_dim, self.dtype = batch, n_heads, head_dim, dtype
        self.n_sink, self.recent, self.norm = n_sink, recent, norm
        # window = w: scores over a history window of w steps (Eq. 3) instead of accumulated ones; only the
        # fused step supports it
        self.window = window
        # q_per_kv = g > 1: grouped-query attention; n_heads counts the K/V heads, query tensors have n_heads * g heads
        self.q_per_kv = int(q_per_kv)
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
        # leading rows the two sets share, per head, as the fused step leaves it (two arrays: one is
        # read while the other is written); synced_cur indexes the valid one
        self.synced = [torch.zeros(batch * n_heads, dtype=torch.int32, device=self.device) for _ in range(2)]
        self.synced_cur = 0
        self._synced_valid = False       # False: the other set holds nothing of the current state
        self.cur = 0
        self.lens: List[int] = [0] * batch
        self._p_dec = B.Params(batch, n_heads, head_dim, dtype, n_sink, recent, self.cap, self.lens, self.budgets,
                               norm=norm, q_per_kv=self.q_per_kv)
        # sized for the fullest cache a decode step may meet (cap - 1 rows plus the new one)
        self._p_dec.set_len([self.cap - 1] * batch)
        nbytes = B.vatp_workspace_bytes(self.ctx, self._p_dec, B.CALL_DECODE_ATTEND_STEP)   # the largest of the decode calls
        self._p_dec.set_len(self.lens)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        self.S_prompt = self.nrm_prompt = None
        if window is not None:
            self.cap_hist = self.cap
            self.hist = torch.zeros(batch, n_heads, window + 2, self.cap_hist, dtype=torch.float32, device=self.device)
            self.hid = [torch.zeros(*shape, dtype=torch.int32, device=self.device) for _ in range(2)]
            self.free = [torch.zeros(batch * n_heads, dtype=torch.int32, device=self.device) for _ in range(2)]
            # low-order parts of the windowed scores (a score is carried in two floats), one array per cache set
            self.S_lo = [torch.zeros(*shape, dtype=torch.float32, device=self.device) for _ in range(2)]
            self.hist_prompt = None
        # The decode calls are made once per generated token: their device pointers are converted to
        # ctypes values once, here, instead of on every call.
        vp = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else None
        self._cp = {name: [vp(x) for x in getattr(self, name)] for name in ("K", "V", "S", "nrm", "pos", "synced")}
        self._cp_kept, self._cp_ws = vp(self.kept_idx), vp(self.ws)
        self._ws_bytes = self.ws.numel()
        self._npos = (ctypes.c_int32 * batch)()
        self._fused_args = {}
        self._lib = B.load()

    def close(self):
        if self._own_ctx and self.ctx is not None:
            B.vatp_destroy(self.ctx)
            self.ctx = None

    # -- prompt pass -----------------------------------------------------------------
    def prefill_score(self, Q, K, V, lens: Sequence[int], stream=None):
        """vatp_prefill_score on [b, H, cap_p, d] prompt tensors (Q: [b, H * q_per_kv, cap_p, d]); results kept in
        S_prompt / nrm_prompt."""
        b, H, cap_p, d = K.shape
        if tuple(Q.shape) != (b, H * self.q_per_kv, cap_p, d):
            raise ValueError("vatp: Q must have n_heads * q_per_kv heads")
        p = B.Params(b, H, d, self.dtype, self.n_sink, self.recent, cap_p, lens, self.budgets, cap_out=self.cap,
                     norm=self.norm, q_per_kv=self.q_per_kv)
        need = B.vatp_workspace_bytes(self.ctx, p, B.CALL_PREFILL_SCORE if self.window is None
                                      else B.CALL_PREFILL_SCORE_WINDOW)
        if getattr(self, "_ws_prompt", None) is None or self._ws_prompt.numel() < need:
            self._ws_prompt = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        if self.S_prompt is None or self.S_prompt.shape != (b, H, cap_p):
            self.S_prompt = torch.empty(b, H, cap_p, dtype=torch.float32, device=self.device)
            self.nrm_prompt = torch.empty(b, H, cap_p, dtype=torch.float32, device=self.device)
        if self.window is None:
            B.vatp_prefill_score(self.ctx, p, Q, K, V, self.S_prompt, self.nrm_prompt, self._ws_prompt, stream)
        else:
            if self.hist_prompt is None or self.hist_prompt.shape != (b, H, self.window + 1, cap_p):
                self.hist_prompt = torch.empty(b, H, self.window + 1, cap_p, dtype=torch.float32, device=self.device)
            B.vatp_prefill_score_window(self.ctx, p, Q, K, V, self.window, self.S_prompt, self.nrm_prompt,
                                        self.hist_prompt, self._ws_prompt, stream)
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
        if self.window is None:
            B.vatp_select_compact(self.ctx, p, K, V, self.S_prompt, self.nrm_prompt, pos_in, self.K[0], self.V[0],
                                  self.S[0], self.nrm[0], self.pos[0], self.kept_idx, None, stream)
        else:
            B.vatp_select_compact_window(self.ctx, p, K, V, self.S_prompt, self.nrm_prompt, pos_in, self.hist_prompt,
                                         self.window, self.K[0], self.V[0], self.S[0], self.nrm[0], self.pos[0],
                                         self.kept_idx, self.hist, self.cap_hist, self.hid[0], self.free[self.synced_cur],
                                         self.S_lo[0], None, stream)
        self.lens = [min(n, bud) for n, bud in zip(self._prompt_lens, self.budgets)]
        self._synced_valid = False

    # -- decode ----------------------------------------------------------------------
    def _new_pos(self, new_pos):
        if self.pos[0] is None or new_pos is None:
            return None
        for i, x in enumerate(new_pos):
            self._npos[i] = x
        return self._npos

    @staticmethod
    def _qkv(q, k, v):
        if not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
            raise ValueError("vatp: tensors must be contiguous")
        return q.data_ptr(), k.data_ptr(), v.data_ptr()            # (plain integers convert to void* arguments)

    def decode_step(self, q, k, v, new_pos: Optional[Sequence[int]], stream=None):
        if self.window is not None:
            raise NotImplementedError("history-window scores go through decode_prune_step")
        c, cp = self.cur, self._cp
        self._p_dec.set_len(self.lens)
        st = self._lib.vatp_decode_step(self.ctx, self._p_dec.ref(), *self._qkv(q, k, v), cp["K"][c], cp["V"][c],
                                        cp["S"][c], cp["nrm"][c], cp["pos"][c], self._new_pos(new_pos), self._cp_ws,
                                        self._ws_bytes, B._stream(stream))
        B._check(st, "vatp_decode_step")
        self.lens = [n + 1 for n in self.lens]

    def prune(self, stream=None):
        c, o, cp = self.cur, 1 - self.cur, self._cp
        self._p_dec.set_len(self.lens)
        st = self._lib.vatp_select_compact(self.ctx, self._p_dec.ref(), cp["K"][c], cp["V"][c], cp["S"][c], cp["nrm"][c],
                                           cp["pos"][c], cp["K"][o], cp["V"][o], cp["S"][o], cp["nrm"][o], cp["pos"][o],
                                           self._cp_kept, None, 0, B._stream(stream))
        B._check(st, "vatp_select_compact")
        self.cur = o
        self.lens = [min(n, bud) for n, bud in zip(self.lens, self.budgets)]
        self._synced_valid = False                    # not tracked by this route

    def decode_prune_step(self, q, k, v, new_pos: Optional[Sequence[int]], out=None, want_kept_idx: bool = True,
                          stream=None):
        """vatp_decode_prune_step: decode_step + prune in two launches, rewriting only the rows that changed."""
        c, o = self.cur, 1 - self.cur
        si, so = self.synced_cur, 1 - self.synced_cur
        if not self._synced_valid:
            self.synced[si].zero_()
            self._synced_valid = True
        self._p_dec.set_len(self.lens)
        cp = self._cp
        if self.window is not None:
            B.vatp_decode_prune_step_window(
                self.ctx, self._p_dec, q, k, v, self.K[c], self.V[c], self.S[c], self.nrm[c], self.pos[c], self.hid[c],
                new_pos, self.K[o], self.V[o], self.S[o], self.nrm[o], self.pos[o], self.hid[o],
                self.kept_idx if want_kept_idx else None, self.synced[si], self.synced[so], self.free[si], self.free[so],
                self.hist, self.S_lo[c], self.S_lo[o], self.window, self.cap_hist, out, self.ws, stream)
            self.cur, self.synced_cur = o, so
            self.lens = [min(n + 1, bud) for n, bud in zip(self.lens, self.budgets)]
            return
        # the arguments that do not change from step to step are laid out once per (cache set, synced array) pair
        args = self._fused_args.get((c, si))
        if args is None:
            args = [self.ctx, self._p_dec.ref(), None, None, None, cp["K"][c], cp["V"][c], cp["S"][c], cp["nrm"][c],
                    cp["pos"][c], None, cp["K"][o], cp["V"][o], cp["S"][o], cp["nrm"][o], cp["pos"][o], None,
                    cp["synced"][si], cp["synced"][so], None, self._cp_ws, self._ws_bytes, None]
            self._fused_args[(c, si)] = args
        args[2], args[3], args[4] = self._qkv(q, k, v)
        args[10] = self._new_pos(new_pos)
        args[16] = self._cp_kept if want_kept_idx else None
        args[17], args[18] = self.synced[si].data_ptr(), self.synced[so].data_ptr()
        args[19] = B._ptr(out)
        args[22] = B._stream(stream)
        st = self._lib.vatp_decode_prune_step(*args)
        if st:
            B._check(st, "vatp_decode_prune_step")
        self.cur, self.synced_cur = o, so
        self.lens = [min(n + 1, bud) for n, bud in zip(self.lens, self.budgets)]
