"""Python face of the float64 CPU oracle -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Loads `liboracle.so` (built from vatp_oracle.c with gcc) through ctypes and offers
  * thin per-head wrappers of the C functions, on numpy float64 arrays;
  * `OracleHead`, the state of one attention head's pruned KV cache carried through the
    prompt pass, the prune and the decode steps in the order the paper's Fig. 2 caption
    gives (score, multiply by the value norm, remove the least important).

Only tests, the smoke check and the bench's CPU-baseline leg may import this module.
It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vatp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no fast-math: IEEE double semantics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None

_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i64 = ctypes.c_int64


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.vatp_oracle_prefill_scores.argtypes = [_f64p, _f64p, _i64, _i64, ctypes.c_double, _f64p, _f64p]
        L.vatp_oracle_prefill_scores.restype = None
        L.vatp_oracle_prefill_scores_from.argtypes = [_f64p, _f64p, _i64, _i64, ctypes.c_double, _i64, _f64p, _f64p]
        L.vatp_oracle_prefill_scores_from.restype = None
        L.vatp_oracle_prefill_window.argtypes = [_f64p, _f64p, _i64, _i64, ctypes.c_double, _i64, _f64p, _f64p, _f64p]
        L.vatp_oracle_prefill_window.restype = _i64
        L.vatp_oracle_row_lse.argtypes = [_f64p, _f64p, _i64, _i64, ctypes.c_double, _f64p, _f64p]
        L.vatp_oracle_row_lse.restype = None
        L.vatp_oracle_prefill_scores_given_lse.argtypes = [_f64p, _f64p, _f64p, _i64, _i64, ctypes.c_double, _f64p]
        L.vatp_oracle_prefill_scores_given_lse.restype = None
        L.vatp_oracle_decode_scores.argtypes = [_f64p, _f64p, _i64, _i64, ctypes.c_double, _f64p, _f64p, _f64p]
        L.vatp_oracle_decode_scores.restype = None
        L.vatp_oracle_attention_output.argtypes = [_f64p, _f64p, _f64p, _i64, _i64, ctypes.c_double, _f64p, _f64p, _f64p]
        L.vatp_oracle_attention_output.restype = None
        L.vatp_oracle_l1norm.argtypes = [_f64p, _i64, _i64, _f64p]
        L.vatp_oracle_l1norm.restype = None
        L.vatp_oracle_vnorm.argtypes = [_f64p, _i64, _i64, ctypes.c_int, _f64p]
        L.vatp_oracle_vnorm.restype = None
        L.vatp_oracle_importance.argtypes = [_f64p, _f64p, _i64, _f64p]
        L.vatp_oracle_importance.restype = None
        L.vatp_oracle_select.argtypes = [_f64p, _i64, _i64, _i64, _i64, _i32p]
        L.vatp_oracle_select.restype = _i64
        L.vatp_oracle_gather_rows.argtypes = [_f64p, _i32p, _i64, _i64, _f64p]
        L.vatp_oracle_gather_rows.restype = None
        L.vatp_oracle_prefill_scores_units.argtypes = [_f64p, _f64p, _i64, _i64, _i64p, _i64,
                                                       ctypes.c_double, _f64p]
        L.vatp_oracle_prefill_scores_units.restype = None
        L.vatp_oracle_decode_prune_units.argtypes = [_f64p, _f64p, _f64p, _f64p, _f64p, _i64, _i64,
                                                     _i64p, _i64, ctypes.c_double, _i64p, _i64, _i64,
                                                     _f64p, _f64p, _f64p, _f64p, _i32p, _i64p]
        L.vatp_oracle_decode_prune_units.restype = None
        L.vatp_oracle_max_threads.argtypes = []
        L.vatp_oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(_f64p)


def default_scale(d: int) -> float:
    """Scaled dot-product attention: logits are <q,k>/sqrt(d)."""
    return 1.0 / float(np.sqrt(np.float64(d)))


def prefill_scores(Q, K, c: Optional[float] = None) -> np.ndarray:
    """S_i = sum_{j>=i} a_i^j over a causal prompt pass (Eq. 1 and Eq. 2). Q, K: [L, d]."""
    Q, K = _f64(Q), _f64(K)
    L, d = Q.shape
    assert K.shape == (L, d)
    S = np.zeros(L, dtype=np.float64)
    scratch = np.zeros(max(L, 1), dtype=np.float64)
    lib().vatp_oracle_prefill_scores(_p(Q), _p(K), L, d, default_scale(d) if c is None else c,
                                     _p(S), _p(scratch))
    return S


def prefill_scores_tail(Q, K, j_start: int, c: Optional[float] = None) -> np.ndarray:
    """Entries i >= j_start of prefill_scores(Q, K), from the query rows j >= j_start only."""
    Q, K = _f64(Q), _f64(K)
    L, d = Q.shape
    S = np.zeros(L, dtype=np.float64)
    scratch = np.zeros(max(L, 1), dtype=np.float64)
    lib().vatp_oracle_prefill_scores_from(_p(Q), _p(K), L, d, default_scale(d) if c is None else c,
                                          int(j_start), _p(S), _p(scratch))
    return S[j_start:]


def prefill_window(Q, K, w: int, c: Optional[float] = None):
    """Eq. 3 after the prompt: (S, P) with S_i = sum of a_i^j over the last w+1 query rows j and
    P [min(L, w+1), L] those attention rows themselves, oldest first.  Q, K: [L, d]."""
    Q, K = _f64(Q), _f64(K)
    L, d = Q.shape
    S = np.zeros(L, dtype=np.float64)
    n_hist = min(L, int(w) + 1)
    P = np.zeros((max(n_hist, 1), max(L, 1)), dtype=np.float64)
    scratch = np.zeros(max(L, 1), dtype=np.float64)
    if L:
        got = lib().vatp_oracle_prefill_window(_p(Q), _p(K), L, d, default_scale(d) if c is None else c, int(w),
                                               _p(S), _p(P), _p(scratch))
        assert got == n_hist
    return S, P[:n_hist, :L]


def prefill_scores_units(Q, K, lens, c: Optional[float] = None) -> np.ndarray:
    """prefill_scores for every unit of Q, K: [units, cap, d] (OpenMP over units). Returns [units, cap]."""
    Q, K = _f64(Q), _f64(K)
    units, cap, d = Q.shape
    lens = np.ascontiguousarray(lens, dtype=np.int64)
    S = np.zeros((units, cap), dtype=np.float64)
    lib().vatp_oracle_prefill_scores_units(_p(Q), _p(K), units, cap, lens.ctypes.data_as(_i64p), d,
                                           default_scale(d) if c is None else c, _p(S))
    return S


def row_lse(Q, K, c: Optional[float] = None) -> np.ndarray:
    """lse_j = ln sum_{i<=j} exp(c <q_j, k_i>): what a fused attention kernel returns per query row."""
    Q, K = _f64(Q), _f64(K)
    L, d = Q.shape
    out = np.zeros(L, dtype=np.float64)
    scratch = np.zeros(max(L, 1), dtype=np.float64)
    lib().vatp_oracle_row_lse(_p(Q), _p(K), L, d, default_scale(d) if c is None else c, _p(out), _p(scratch))
    return out


def prefill_scores_given_lse(Q, K, lse, c: Optional[float] = None) -> np.ndarray:
    """S_i = sum_{j>=i} exp(c <q_j,k_i> - lse_j): Eq. 2 after the prompt with the row normalisers given."""
    Q, K, lse = _f64(Q), _f64(K), _f64(lse)
    L, d = Q.shape
    S = np.zeros(L, dtype=np.float64)
    lib().vatp_oracle_prefill_scores_given_lse(_p(Q), _p(K), _p(lse), L, d, default_scale(d) if c is None else c, _p(S))
    return S


def decode_scores(q, K, S, c: Optional[float] = None):
    """One decode step of Eq. 2. Returns (S + a, a) for the n rows of K."""
    q, K = _f64(q), _f64(K)
    n, d = K.shape
    S = _f64(S).copy()
    assert S.shape == (n,) and q.shape == (d,)
    a = np.zeros(n, dtype=np.float64)
    scratch = np.zeros(max(n, 1), dtype=np.float64)
    lib().vatp_oracle_decode_scores(_p(q), _p(K), n, d, default_scale(d) if c is None else c,
                                    _p(S), _p(a), _p(scratch))
    return S, a


def attention_output(q, K, V, c: Optional[float] = None):
    """Eq. 1 for one query: (sum_r a_r V_r, sum_r a_r |V_r|) over the n rows of K, V."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    n, d = K.shape
    out, abs_out = np.zeros(d), np.zeros(d)
    scratch = np.zeros(max(n, 1), dtype=np.float64)
    lib().vatp_oracle_attention_output(_p(q), _p(K), _p(V), n, d, default_scale(d) if c is None else c,
                                       _p(out), _p(abs_out), _p(scratch))
    return out, abs_out


def prefill_scores_group(Qg, K, c: Optional[float] = None) -> np.ndarray:
    """Grouped-query attention (Limitations section, paragraph on GQA): the g query heads that share one
    key/value head each attend on their own (Eq. 1, 2); the token score of the shared head is the mean of
    their accumulated scores.  Qg: [g, L, d], K: [L, d]."""
    Qg = _f64(Qg)
    g = Qg.shape[0]
    S = np.zeros(Qg.shape[1], dtype=np.float64)
    for r in range(g):
        S += prefill_scores(Qg[r], K, c)
    return S / g


def prefill_window_group(Qg, K, w: int, c: Optional[float] = None):
    """prefill_window with g query heads on one K/V head: (S, P), both means over the group (Eq. 3 applied to
    the group-averaged attention weights).  Qg: [g, L, d]."""
    Qg = _f64(Qg)
    g = Qg.shape[0]
    S, P = prefill_window(Qg[0], K, w, c)
    for r in range(1, g):
        s_r, p_r = prefill_window(Qg[r], K, w, c)
        S = S + s_r
        P = P + p_r
    return S / g, P / g


def prefill_scores_group_units(Qg, K, lens, c: Optional[float] = None) -> np.ndarray:
    """prefill_scores_group for many K/V heads at once (OpenMP over query heads).
    Qg: [units, g, cap, d], K: [units, cap, d]. Returns [units, cap]."""
    Qg, K = _f64(Qg), _f64(K)
    units, g, cap, d = Qg.shape
    lens = np.asarray(lens, dtype=np.int64)
    S_q = prefill_scores_units(Qg.reshape(units * g, cap, d), np.repeat(K, g, axis=0), np.repeat(lens, g), c)
    S = np.zeros((units, cap), dtype=np.float64)
    for r in range(g):                     # same order of additions as prefill_scores_group
        S += S_q.reshape(units, g, cap)[:, r]
    return S / g


def decode_scores_group(qg, K, S, c: Optional[float] = None):
    """One decode step with g query heads on one key/value head: (S + a, a) with a the mean over the
    group of the heads' attention weights (each head has its own softmax).  qg: [g, d]."""
    qg, K = _f64(qg), _f64(K)
    g, n = qg.shape[0], K.shape[0]
    a = np.zeros(n, dtype=np.float64)
    for r in range(g):
        _, ar = decode_scores(qg[r], K, np.zeros(n), c)
        a += ar
    a /= g
    return _f64(S) + a, a


def l1norm(V) -> np.ndarray:
    V = _f64(V)
    n, d = V.shape
    out = np.zeros(n, dtype=np.float64)
    lib().vatp_oracle_l1norm(_p(V), n, d, _p(out))
    return out


def vnorm(V, kind: int = 0) -> np.ndarray:
    """Row norms for the ablation of Table 2: kind 0 = l1, 1 = l2, 2 = l-infinity; 3 = all ones, the
    attention-only ranking the paper compares against (H2O)."""
    V = _f64(V)
    n, d = V.shape
    out = np.zeros(n, dtype=np.float64)
    lib().vatp_oracle_vnorm(_p(V), n, d, int(kind), _p(out))
    return out


def importance(S, nrm) -> np.ndarray:
    """Eq. 4: the score times the norm of the value row."""
    S, nrm = _f64(S), _f64(nrm)
    out = np.zeros_like(S)
    lib().vatp_oracle_importance(_p(S), _p(nrm), S.shape[0], _p(out))
    return out


def select(I, B: int, F: int, R: int) -> np.ndarray:
    """Ascending surviving row indices (int32). Raises ValueError if B < F + R."""
    I = _f64(I)
    n = I.shape[0]
    kept = np.zeros(max(min(n, B), 1), dtype=np.int32)
    nk = lib().vatp_oracle_select(_p(I), n, B, F, R, kept.ctypes.data_as(_i32p))
    if nk < 0:
        raise ValueError("budget smaller than forced prefix + recent window")
    return kept[:nk].copy()


def gather_rows(x, kept) -> np.ndarray:
    x = _f64(x)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    width = int(np.prod(x.shape[1:], dtype=np.int64))        # also right for a cache with no rows
    flat = x.reshape(x.shape[0], width)
    out = np.zeros((kept.shape[0], flat.shape[1]), dtype=np.float64)
    lib().vatp_oracle_gather_rows(_p(flat), kept.ctypes.data_as(_i32p), kept.shape[0],
                                  flat.shape[1], _p(out))
    return out.reshape((kept.shape[0],) + x.shape[1:])


def threshold_and_slack(I, n: int, B: int, F: int, R: int):
    """tau = the smallest importance among the oracle's importance-selected candidates,
    or None when nothing is selected by importance (n <= B or B == F + R)."""
    if n <= B or B - F - R <= 0:
        return None
    cand = np.sort(np.asarray(I[F:n - R], dtype=np.float64))[::-1]
    return float(cand[B - F - R - 1])


class OracleHead:
    """Pruned KV cache of one head, stepped exactly as the method prescribes.

    prefill(Q, K, V)    full causal pass over the prompt, norms, no pruning yet
    prune(B, F, R)      Eq. 4 importance -> budgeted selection -> compaction
    append_and_score()  the new token's row joins the cache, its query attends over all
                        rows (itself included) and the accumulated scores grow (Eq. 2)
    `prune` accepts a forced surviving set so that a harness can re-align this state with
    another implementation after an admissible near-tie difference.
    """

    def __init__(self, d: int, c: Optional[float] = None, norm_kind: int = 0, window: Optional[int] = None,
                 group: int = 1):
        self.d = d
        self.norm_kind = norm_kind
        # group = g > 1: grouped-query attention, g query heads on this key/value head; queries then come as
        # [g, L, d] (prompt) and [g, d] (decode step) and scores are means over the group
        self.group = group
        # window = w: scores are sums over the last w+1 steps only (Eq. 3); `hist` then holds those
        # steps' attention rows (oldest first, one entry per cached row) and S is their plain sum
        self.window = window
        self.hist: List[np.ndarray] = []
        self.c = default_scale(d) if c is None else c
        self.K = np.zeros((0, d))
        self.V = np.zeros((0, d))
        self.S = np.zeros(0)
        self.nrm = np.zeros(0)
        self.pos = np.zeros(0, dtype=np.int64)

    @property
    def n(self) -> int:
        return self.K.shape[0]

    def prefill(self, Q, K, V):
        self.K, self.V = _f64(K).copy(), _f64(V).copy()
        if self.group > 1 and self.window is not None:
            self.S, P = prefill_window_group(Q, self.K, self.window, self.c)
            self.hist = [row.copy() for row in P]
        elif self.group > 1:
            self.S = prefill_scores_group(Q, self.K, self.c)
        elif self.window is None:
            self.S = prefill_scores(Q, self.K, self.c)
        else:
            self.S, P = prefill_window(Q, self.K, self.window, self.c)
            self.hist = [row.copy() for row in P]
        self.nrm = l1norm(self.V) if self.norm_kind == 0 else vnorm(self.V, self.norm_kind)
        self.pos = np.arange(self.K.shape[0], dtype=np.int64)

    def importance(self) -> np.ndarray:
        return importance(self.S, self.nrm)

    def prune(self, B: int, F: int, R: int, forced: Optional[Sequence[int]] = None) -> np.ndarray:
        kept = select(self.importance(), B, F, R) if forced is None \
            else np.ascontiguousarray(forced, dtype=np.int32)
        self.K = gather_rows(self.K, kept)
        self.V = gather_rows(self.V, kept)
        self.S = gather_rows(self.S, kept)
        self.nrm = gather_rows(self.nrm, kept)
        self.pos = self.pos[kept]
        self.hist = [row[kept] for row in self.hist]
        return kept

    def append_and_score(self, q, k, v, new_pos: int) -> np.ndarray:
        self.K = np.concatenate([self.K, _f64(k)[None, :]], axis=0)
        self.V = np.concatenate([self.V, _f64(v)[None, :]], axis=0)
        self.S = np.concatenate([self.S, np.zeros(1)])
        new_row = _f64(v)[None, :]
        self.nrm = np.concatenate([self.nrm, l1norm(new_row) if self.norm_kind == 0 else vnorm(new_row, self.norm_kind)])
        self.pos = np.concatenate([self.pos, np.array([new_pos], dtype=np.int64)])
        if self.group > 1:
            self.S, a = decode_scores_group(q, self.K, self.S, self.c)
        else:
            self.S, a = decode_scores(q, self.K, self.S, self.c)
        if self.window is not None:
            # the new row was not there at earlier steps; the oldest step leaves the window
            self.hist = [np.concatenate([row, np.zeros(1)]) for row in self.hist] + [a.copy()]
            self.hist = self.hist[-(self.window + 1):]
            self.S = np.sum(np.stack(self.hist), axis=0)
        return a


def max_threads() -> int:
    return int(lib().vatp_oracle_max_threads())
