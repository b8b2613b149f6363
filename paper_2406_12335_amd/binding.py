"""ctypes binding of libvatp.so: argument marshalling only.

Every function has the name and the argument order of the C entry point it calls
(include/vatp.h); torch tensors stand for device pointers, Python int lists for the host
arrays.  Nothing is computed here, and there is no fallback: if the HIP library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvatp.so")

VATP_F32, VATP_BF16 = 0, 1
NORM_L1, NORM_L2, NORM_LINF, NORM_NONE = 0, 1, 2, 3
CALL_PREFILL_SCORE, CALL_DECODE_STEP, CALL_SELECT_COMPACT, CALL_DECODE_ATTEND_STEP, CALL_DECODE_PRUNE_STEP = 0, 1, 2, 3, 4
CALL_PREFILL_SCORE_WINDOW = 5
VATP_MAX_BATCH, VATP_MAX_UNITS, VATP_MAX_GROUP = 256, 16384, 16
VATP_STATIC_SCRATCH_BYTES = 16777216
OK, E_NULL, E_SHAPE, E_DTYPE, E_BUDGET, E_WORKSPACE, E_DEVICE = 0, -1, -2, -3, -4, -5, -6

EXPORTS = ("vatp_create", "vatp_destroy", "vatp_strerror", "vatp_validate", "vatp_workspace_bytes",
           "vatp_prefill_score", "vatp_prefill_score_lse", "vatp_decode_step", "vatp_decode_attend_step", "vatp_select_compact",
           "vatp_decode_prune_step", "vatp_decode_prune_step_static", "vatp_prefill_score_window", "vatp_select_compact_window",
           "vatp_decode_prune_step_window")


class VatpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


class _Params(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("n_sink", ctypes.c_int32), ("recent", ctypes.c_int32),
                ("cap", ctypes.c_int32), ("cap_out", ctypes.c_int32), ("scale", ctypes.c_float),
                ("len", ctypes.POINTER(ctypes.c_int32)), ("budget", ctypes.POINTER(ctypes.c_int32)),
                ("norm", ctypes.c_int32), ("q_per_kv", ctypes.c_int32)]


_lib = None
_vp = ctypes.c_void_p


def load() -> ctypes.CDLL:
    """Loads the built library.  It is built first when there is none, or when the one that is there was built
    from other sources than the present ones (a digest of sources, headers and flags is kept beside it)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if LIB_PATH == _build.LIB and not _build.is_current():
        _build.build_library()
    elif not os.path.exists(LIB_PATH):
        raise FileNotFoundError("vatp: no library at %s" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    pp = ctypes.POINTER(_Params)
    L.vatp_create.argtypes = [ctypes.POINTER(_vp), ctypes.c_int]
    L.vatp_create.restype = ctypes.c_int
    L.vatp_destroy.argtypes = [_vp]
    L.vatp_destroy.restype = None
    L.vatp_strerror.argtypes = [ctypes.c_int]
    L.vatp_strerror.restype = ctypes.c_char_p
    L.vatp_validate.argtypes = [pp, ctypes.c_int]
    L.vatp_validate.restype = ctypes.c_int
    L.vatp_workspace_bytes.argtypes = [_vp, pp, ctypes.c_int]
    L.vatp_workspace_bytes.restype = ctypes.c_size_t
    L.vatp_prefill_score.argtypes = [_vp, pp] + [_vp] * 5 + [_vp, ctypes.c_size_t, _vp]
    L.vatp_prefill_score.restype = ctypes.c_int
    L.vatp_prefill_score_lse.argtypes = [_vp, pp] + [_vp] * 6 + [_vp, ctypes.c_size_t, _vp]
    L.vatp_prefill_score_lse.restype = ctypes.c_int
    L.vatp_decode_step.argtypes = [_vp, pp] + [_vp] * 8 + [ctypes.POINTER(ctypes.c_int32), _vp, ctypes.c_size_t, _vp]
    L.vatp_decode_step.restype = ctypes.c_int
    L.vatp_decode_attend_step.argtypes = [_vp, pp] + [_vp] * 8 + [ctypes.POINTER(ctypes.c_int32), _vp, _vp, ctypes.c_size_t,
                                                          _vp]
    L.vatp_decode_attend_step.restype = ctypes.c_int
    L.vatp_decode_prune_step.argtypes = [_vp, pp] + [_vp] * 8 + [ctypes.POINTER(ctypes.c_int32)] + [_vp] * 9 + \
        [_vp, ctypes.c_size_t, _vp]
    L.vatp_decode_prune_step.restype = ctypes.c_int
    L.vatp_decode_prune_step_static.argtypes = [_vp, pp] + [_vp] * 8 + [ctypes.POINTER(ctypes.c_int32)] + [_vp] * 9 + [_vp]
    L.vatp_decode_prune_step_static.restype = ctypes.c_int
    i32, i32p = ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
    L.vatp_prefill_score_window.argtypes = [_vp, pp, _vp, _vp, _vp, i32, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
    L.vatp_prefill_score_window.restype = ctypes.c_int
    L.vatp_select_compact_window.argtypes = [_vp, pp] + [_vp] * 6 + [i32] + [_vp] * 7 + [i32, _vp, _vp, _vp] + \
        [_vp, ctypes.c_size_t, _vp]
    L.vatp_select_compact_window.restype = ctypes.c_int
    L.vatp_decode_prune_step_window.argtypes = [_vp, pp] + [_vp] * 9 + [i32p] + [_vp] * 14 + [i32, i32, _vp] + \
        [_vp, ctypes.c_size_t, _vp]
    L.vatp_decode_prune_step_window.restype = ctypes.c_int
    L.vatp_select_compact.argtypes = [_vp, pp] + [_vp] * 11 + [_vp, ctypes.c_size_t, _vp]
    L.vatp_select_compact.restype = ctypes.c_int
    _lib = L
    return L


def strerror(status: int) -> str:
    return load().vatp_strerror(int(status)).decode()


class Params:
    """Host-side mirror of vatp_params; keeps the int arrays alive while a call runs."""

    def __init__(self, batch: int, n_heads: int, head_dim: int, dtype, n_sink: int, recent: int,
                 cap: int, len: Sequence[int], budget: Optional[Sequence[int]] = None,
                 cap_out: int = 0, scale: float = 0.0, norm: int = 0, q_per_kv: int = 0):
        if isinstance(dtype, torch.dtype):
            dtype = {torch.float32: VATP_F32, torch.bfloat16: VATP_BF16}.get(dtype, -1)
        self._len = (ctypes.c_int32 * max(1, batch))(*list(len)) if len is not None else None
        self._budget = (ctypes.c_int32 * max(1, batch))(*list(budget)) if budget is not None else None
        self.c = _Params(batch, n_heads, head_dim, int(dtype), n_sink, recent, cap, cap_out, scale,
                         ctypes.cast(self._len, ctypes.POINTER(ctypes.c_int32)) if self._len is not None else None,
                         ctypes.cast(self._budget, ctypes.POINTER(ctypes.c_int32)) if self._budget is not None else None,
                         int(norm), int(q_per_kv))

    def set_len(self, len: Sequence[int]) -> None:
        for i, v in enumerate(len):
            self._len[i] = int(v)

    def ref(self):
        return ctypes.byref(self.c)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("vatp: tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)     # (handle of the current stream without a Stream object)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        if _raw_stream is not None:
            return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(st: int, where: str) -> None:
    if st != OK:
        raise VatpError(st, where)


def vatp_create(device: int = 0) -> ctypes.c_void_p:
    ctx = _vp()
    _check(load().vatp_create(ctypes.byref(ctx), int(device)), "vatp_create")
    return ctx


def vatp_destroy(ctx) -> None:
    load().vatp_destroy(ctx)


def vatp_validate(p: Params, which_call: int) -> int:
    return int(load().vatp_validate(p.ref(), which_call))


def vatp_workspace_bytes(ctx, p: Params, which_call: int) -> int:
    return int(load().vatp_workspace_bytes(ctx, p.ref(), which_call))


def vatp_prefill_score(ctx, p: Params, Q, K, V, S, nrm, ws, stream=None) -> None:
    _check(load().vatp_prefill_score(ctx, p.ref(), _ptr(Q), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm),
                                     _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                     _stream(stream)), "vatp_prefill_score")


def vatp_prefill_score_lse(ctx, p: Params, Q, K, V, lse, S, nrm, ws, stream=None) -> None:
    _check(load().vatp_prefill_score_lse(ctx, p.ref(), _ptr(Q), _ptr(K), _ptr(V), _ptr(lse), _ptr(S), _ptr(nrm),
                                         _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                         _stream(stream)), "vatp_prefill_score_lse")


def vatp_decode_step(ctx, p: Params, q, k, v, K, V, S, nrm, pos, new_pos: Optional[Sequence[int]], ws,
                     stream=None) -> None:
    npos = (ctypes.c_int32 * len(new_pos))(*[int(x) for x in new_pos]) if new_pos is not None else None
    _check(load().vatp_decode_step(ctx, p.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm),
                                   _ptr(pos), npos, _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "vatp_decode_step")


def vatp_decode_attend_step(ctx, p: Params, q, k, v, K, V, S, nrm, pos, new_pos: Optional[Sequence[int]], out, ws,
                            stream=None) -> None:
    npos = (ctypes.c_int32 * len(new_pos))(*[int(x) for x in new_pos]) if new_pos is not None else None
    _check(load().vatp_decode_attend_step(ctx, p.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(K), _ptr(V), _ptr(S),
                                          _ptr(nrm), _ptr(pos), npos, _ptr(out), _ptr(ws),
                                          ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "vatp_decode_attend_step")


def vatp_decode_prune_step(ctx, p: Params, q, k, v, K, V, S, nrm, pos, new_pos: Optional[Sequence[int]], K_out, V_out,
                           S_out, nrm_out, pos_out, kept_idx, synced_in, synced_out, out, ws, stream=None) -> None:
    npos = (ctypes.c_int32 * len(new_pos))(*[int(x) for x in new_pos]) if new_pos is not None else None
    _check(load().vatp_decode_prune_step(ctx, p.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm),
                                         _ptr(pos), npos, _ptr(K_out), _ptr(V_out), _ptr(S_out), _ptr(nrm_out),
                                         _ptr(pos_out), _ptr(kept_idx), _ptr(synced_in), _ptr(synced_out), _ptr(out),
                                         _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                         _stream(stream)), "vatp_decode_prune_step")


def vatp_decode_prune_step_static(ctx, p: Params, q, k, v, K, V, S, nrm, pos, new_pos: Optional[Sequence[int]], K_out,
                                  V_out, S_out, nrm_out, pos_out, kept_idx, synced_in, synced_out, out,
                                  stream=None) -> None:
    npos = (ctypes.c_int32 * len(new_pos))(*[int(x) for x in new_pos]) if new_pos is not None else None
    _check(load().vatp_decode_prune_step_static(ctx, p.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(K), _ptr(V), _ptr(S),
                                                _ptr(nrm), _ptr(pos), npos, _ptr(K_out), _ptr(V_out), _ptr(S_out),
                                                _ptr(nrm_out), _ptr(pos_out), _ptr(kept_idx), _ptr(synced_in),
                                                _ptr(synced_out), _ptr(out), _stream(stream)),
           "vatp_decode_prune_step_static")


def _nbytes(ws) -> int:
    return ws.numel() * ws.element_size() if ws is not None else 0


def vatp_prefill_score_window(ctx, p: Params, Q, K, V, window: int, S, nrm, hist, ws, stream=None) -> None:
    _check(load().vatp_prefill_score_window(ctx, p.ref(), _ptr(Q), _ptr(K), _ptr(V), int(window), _ptr(S), _ptr(nrm),
                                            _ptr(hist), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vatp_prefill_score_window")


def vatp_select_compact_window(ctx, p: Params, K, V, S, nrm, pos, hist, window: int, K_out, V_out, S_out, nrm_out,
                               pos_out, kept_idx, hist_out, cap_hist: int, hid_out, free_out, S_lo_out, ws=None,
                               stream=None) -> None:
    _check(load().vatp_select_compact_window(ctx, p.ref(), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm), _ptr(pos), _ptr(hist),
                                             int(window), _ptr(K_out), _ptr(V_out), _ptr(S_out), _ptr(nrm_out),
                                             _ptr(pos_out), _ptr(kept_idx), _ptr(hist_out), int(cap_hist),
                                             _ptr(hid_out), _ptr(free_out), _ptr(S_lo_out), _ptr(ws), _nbytes(ws),
                                             _stream(stream)),
           "vatp_select_compact_window")


def vatp_decode_prune_step_window(ctx, p: Params, q, k, v, K, V, S, nrm, pos, hid, new_pos: Sequence[int], K_out,
                                  V_out, S_out, nrm_out, pos_out, hid_out, kept_idx, synced_in, synced_out, free_in,
                                  free_out, hist, S_lo, S_lo_out, window: int, cap_hist: int, out, ws,
                                  stream=None) -> None:
    npos = (ctypes.c_int32 * len(new_pos))(*[int(x) for x in new_pos]) if new_pos is not None else None
    _check(load().vatp_decode_prune_step_window(
        ctx, p.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm), _ptr(pos), _ptr(hid), npos,
        _ptr(K_out), _ptr(V_out), _ptr(S_out), _ptr(nrm_out), _ptr(pos_out), _ptr(hid_out), _ptr(kept_idx),
        _ptr(synced_in), _ptr(synced_out), _ptr(free_in), _ptr(free_out), _ptr(hist), _ptr(S_lo), _ptr(S_lo_out),
        int(window), int(cap_hist),
        _ptr(out), _ptr(ws), _nbytes(ws), _stream(stream)), "vatp_decode_prune_step_window")


def vatp_select_compact(ctx, p: Params, K, V, S, nrm, pos, K_out, V_out, S_out, nrm_out, pos_out, kept_idx,
                        ws=None, stream=None) -> None:
    _check(load().vatp_select_compact(ctx, p.ref(), _ptr(K), _ptr(V), _ptr(S), _ptr(nrm), _ptr(pos), _ptr(K_out),
                                      _ptr(V_out), _ptr(S_out), _ptr(nrm_out), _ptr(pos_out), _ptr(kept_idx),
                                      _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                      _stream(stream)), "vatp_select_compact")
