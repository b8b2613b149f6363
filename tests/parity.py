"""Harness that walks the HIP path and the CPU oracle through the same trajectory.

Comparison rules
  scores        |gpu - oracle| <= rtol * |oracle| + 1e-12, rtol = 1e-5 (fp32) / 1e-3 (bf16)
  kept sets     identical, except that a difference is admitted when it lies inside the
                oracle's own near-tie band: every candidate the GPU kept has oracle
                importance >= tau (1 - rtol) and every candidate it dropped has
                <= tau (1 + rtol), tau being the oracle's weakest importance-selected
                candidate.  After an admitted difference the oracle state is re-aligned to
                the GPU's kept set (and the event counted), since both continue from
                different caches otherwise.
  compaction    rows, scores, norms and positions of the survivors equal their source rows
                bit for bit (checked on the GPU's own buffers).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle import vatp_oracle as orc  # noqa: F401 (also used as parity.orc)
from paper_2406_12335_amd.runner import PrunedKVCache

ATOL = 1e-12
WINDOW_ABS = 2.0 ** -36       # windowed scores: absolute tolerance as a fraction of the largest score the row has had


def rtol_for(dtype: torch.dtype) -> float:
    return 1e-5 if dtype == torch.float32 else 1e-3


def assert_scores_close(got, want, rtol, what="", atol=0.0):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    bound = rtol * np.abs(want) + ATOL + atol
    if not np.all(err <= bound):
        i = int(np.argmax(err / bound))
        raise AssertionError("%s: %d of %d beyond tolerance; worst at %d: got %.9g want %.9g (rel %.3g)" % (
            what, int(np.sum(err > bound)), err.size, i, got[i], want[i], err[i] / max(abs(want[i]), 1e-300)))
    floor = np.maximum(1e-300, np.asarray(atol, dtype=np.float64) / rtol)   # below this magnitude the absolute part of the bound governs
    return float(np.max(err / np.maximum(np.abs(want), floor))) if err.size else 0.0


def check_kept_set(kept_gpu: np.ndarray, I_oracle: np.ndarray, n: int, B: int, F: int, R: int,
                   rtol: float, atol: float = 0.0) -> Tuple[bool, np.ndarray]:
    """Returns (identical, oracle_kept). Raises if the GPU set is outside the near-tie band.
    atol widens the band by an absolute amount of importance on either side (history-window scores: see
    run_trajectory; it is many orders of magnitude below the relative band in every case met so far)."""
    kept_or = orc.select(I_oracle, B, F, R)
    assert len(kept_gpu) == len(kept_or) == min(n, B), "kept count differs from the budget"
    if np.array_equal(kept_gpu, kept_or):
        return True, kept_or
    assert np.all(np.diff(kept_gpu) > 0), "kept indices not strictly ascending"
    gset = set(kept_gpu.tolist())
    assert set(range(F)) <= gset and set(range(n - R, n)) <= gset, "protected rows missing"
    tau = orc.threshold_and_slack(I_oracle, n, B, F, R)
    assert tau is not None
    cand = np.arange(F, n - R)
    in_gpu = np.isin(cand, kept_gpu)
    Ic = I_oracle[cand]
    bad_kept = cand[in_gpu & (Ic < tau * (1 - rtol) - 2 * atol)]
    bad_drop = cand[~in_gpu & (Ic > tau * (1 + rtol) + 2 * atol)]
    if len(bad_kept) or len(bad_drop):
        raise AssertionError("kept set differs outside the near-tie band: wrongly kept %s, wrongly dropped %s "
                             "(tau=%.9g)" % (bad_kept[:8].tolist(), bad_drop[:8].tolist(), tau))
    return False, kept_or


@dataclasses.dataclass
class TrajectoryReport:
    units_checked: int = 0
    prune_events: int = 0
    admitted_near_ties: int = 0
    max_rel_err_prefill: float = 0.0
    max_rel_err_decode: float = 0.0


def _unit_rows(t: torch.Tensor, b: int, h: int, n: int) -> np.ndarray:
    return t[b, h, :n].detach().to(torch.float64).cpu().numpy()


def _vec(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def run_trajectory(inp, device, units: Optional[Sequence[Tuple[int, int]]] = None, steps: Optional[int] = None,
                   n_sink: Optional[int] = None, check_every: int = 1, cap_cache: Optional[int] = None,
                   prefill_oracle: Optional[Dict[Tuple[int, int], np.ndarray]] = None, norm_kind: int = 0,
                   fused: bool = False, window: Optional[int] = None) -> TrajectoryReport:
    """Prompt pass -> prune -> decode/prune steps on the GPU, mirrored by OracleHead on the chosen units.

    The oracle's state never takes a value from the GPU: its prompt scores are computed here, by the oracle, for
    every chosen unit -- or handed in through prefill_oracle ({unit: the oracle's S for that unit}) by a test
    that has already computed them, so that an expensive prompt pass is not run twice.  Either way the GPU's
    prompt scores are compared with them element by element, and the prompt prune is judged on the oracle's.

    fused: every decode step and its prune go through vatp_decode_prune_step instead of
    vatp_decode_step + vatp_select_compact; the state after each step is compared with the oracle's.
    window = w: scores over a history window of w steps (Eq. 3; fused steps only).  The GPU carries such a
    score in two floats, adding each new weight and later subtracting the same float by error-free
    transformations, so the relative tolerance holds as for accumulated scores; the only absolute term is
    WINDOW_ABS = 2^-36 of the largest score THAT ROW has ever had (the carried sum loses at most 2^-47 of
    its value per step: room for thousands of steps), which matters only for a row whose score has fallen
    by more than nine orders of magnitude."""
    cfg = inp.cfg
    b, H, d = cfg.batch, cfg.n_heads, cfg.head_dim
    grp = cfg.q_per_kv                       # > 1: grouped queries, query heads h*grp .. h*grp+grp-1 on K/V head h
    F = cfg.n_sink_keep if n_sink is None else n_sink
    R = cfg.recent
    T = cfg.decode_steps if steps is None else steps
    rtol = rtol_for(cfg.torch_dtype())
    units = [(bb, hh) for bb in range(b) for hh in range(H)] if units is None else list(units)
    rep = TrajectoryReport(units_checked=len(units))

    dev = lambda t: t.to(device)
    Q, K, V = dev(inp.Q), dev(inp.K), dev(inp.V)
    qd, kd, vd = dev(inp.qd), dev(inp.kd), dev(inp.vd)
    assert window is None or fused
    cache = PrunedKVCache(b, H, d, cfg.torch_dtype(), F, R, inp.budgets, device, cap_cache=cap_cache, norm=norm_kind,
                          window=window, q_per_kv=grp)

    def q_of(t: torch.Tensor, bb: int, hh: int) -> np.ndarray:
        """Decode query of unit (bb, hh): [d], or [grp, d] for grouped queries."""
        return _vec(t[bb, hh]) if grp == 1 else _vec(t[bb, hh * grp:(hh + 1) * grp])

    row_max = {}                             # windowed scores: largest oracle score every cached row has had, per unit
    try:
        cache.prefill_score(Q, K, V, inp.lens)
        torch.cuda.synchronize()
        heads: Dict[Tuple[int, int], orc.OracleHead] = {}
        # oracle prompt pass for the chosen units (OpenMP over units)
        Lmax = max(inp.lens)
        Kh = np.stack([_unit_rows(inp.K, bb, hh, Lmax) for bb, hh in units])
        S_or = None
        have = prefill_oracle is not None and window is None
        if have:
            assert all(u in prefill_oracle for u in units), "prefill_oracle must cover every chosen unit"
        if grp == 1:
            if window is not None or not have:
                Qh = np.stack([_unit_rows(inp.Q, bb, hh, Lmax) for bb, hh in units])
            if window is None and not have:
                S_or = orc.prefill_scores_units(Qh, Kh, [inp.lens[bb] for bb, _ in units])
        else:
            Qg = np.stack([np.stack([_unit_rows(inp.Q, bb, hh * grp + r, Lmax) for r in range(grp)]) for bb, hh in units])
            if window is None and not have:
                S_or = orc.prefill_scores_group_units(Qg, Kh, [inp.lens[bb] for bb, _ in units])
        for ui, (bb, hh) in enumerate(units):
            L = inp.lens[bb]
            o = orc.OracleHead(d, norm_kind=norm_kind, window=window, group=grp)
            o.K, o.V = Kh[ui, :L].copy(), _unit_rows(inp.V, bb, hh, L)
            o.nrm = orc.vnorm(o.V, norm_kind)
            o.pos = np.arange(L, dtype=np.int64)
            S_gpu = _unit_rows(cache.S_prompt, bb, hh, L)
            if window is not None:
                o.S, P = orc.prefill_window(Qh[ui, :L], Kh[ui, :L], window) if grp == 1 \
                    else orc.prefill_window_group(Qg[ui, :, :L], Kh[ui, :L], window)
                o.hist = [row.copy() for row in P]
                row_max[(bb, hh)] = o.S.copy()
                e = assert_scores_close(S_gpu, o.S, rtol, "windowed prefill S unit (%d,%d)" % (bb, hh))
                rep.max_rel_err_prefill = max(rep.max_rel_err_prefill, e)
            else:
                o.S = np.array(prefill_oracle[(bb, hh)][:L], dtype=np.float64) if have else S_or[ui, :L].copy()
                e = assert_scores_close(S_gpu, o.S, rtol, "prefill S unit (%d,%d)" % (bb, hh))
                rep.max_rel_err_prefill = max(rep.max_rel_err_prefill, e)
            assert_scores_close(_unit_rows(cache.nrm_prompt, bb, hh, L), o.nrm, rtol, "nrm unit (%d,%d)" % (bb, hh))
            heads[(bb, hh)] = o

        def check_prune(src_K, src_V, src_S, src_nrm, src_pos, n_before: List[int]):
            torch.cuda.synchronize()
            c = cache.cur
            for (bb, hh), o in heads.items():
                n, Bq = n_before[bb], inp.budgets[bb]
                nk = min(n, Bq)
                kept_gpu = cache.kept_idx[bb, hh, :nk].cpu().numpy()
                same, _ = check_kept_set(kept_gpu, o.importance(), n, Bq, F, R, rtol)
                rep.prune_events += 1
                rep.admitted_near_ties += 0 if same else 1
                o.prune(Bq, F, R, forced=kept_gpu)
                if window is not None:
                    row_max[(bb, hh)] = row_max[(bb, hh)][kept_gpu]
                idx = torch.from_numpy(kept_gpu.astype(np.int64)).to(device)
                assert torch.equal(cache.K[c][bb, hh, :nk], src_K[bb, hh].index_select(0, idx)), "K rows differ"
                assert torch.equal(cache.V[c][bb, hh, :nk], src_V[bb, hh].index_select(0, idx)), "V rows differ"
                assert torch.equal(cache.S[c][bb, hh, :nk], src_S[bb, hh].index_select(0, idx)), "S entries differ"
                assert torch.equal(cache.nrm[c][bb, hh, :nk], src_nrm[bb, hh].index_select(0, idx)), "nrm differ"
                if src_pos is not None:
                    assert torch.equal(cache.pos[c][bb, hh, :nk], src_pos[bb, hh].index_select(0, idx)), "pos differ"
                    assert np.array_equal(cache.pos[c][bb, hh, :nk].cpu().numpy(), o.pos), "positions differ from oracle"

        n_before = list(inp.lens)
        cache.prune_prompt(K, V)
        check_prune(K, V, cache.S_prompt, cache.nrm_prompt, cache._pos_prompt, n_before)

        def check_fused_step(t, n_before: List[int], do_check: bool):
            torch.cuda.synchronize()
            c = cache.cur
            for (bb, hh), o in heads.items():
                n, Bq = n_before[bb], inp.budgets[bb]
                nk = min(n, Bq)
                kept_gpu = cache.kept_idx[bb, hh, :nk].cpu().numpy()
                # windowed scores: per-row absolute term (see the docstring), carried into the importance by the
                # row's own norm; the band around the threshold takes the largest such term among the candidates
                atol_rows, atol_I = None, 0.0
                if window is not None:
                    rm = np.maximum(np.append(row_max[(bb, hh)], 0.0), o.S)        # (the appended row starts at 0)
                    atol_rows = WINDOW_ABS * rm
                    cand = slice(F, max(F, n - R))
                    atol_I = float(np.max(atol_rows[cand] * o.nrm[cand])) if n - R > F else 0.0
                same, _ = check_kept_set(kept_gpu, o.importance(), n, Bq, F, R, rtol, atol=atol_I)
                rep.prune_events += 1
                rep.admitted_near_ties += 0 if same else 1
                o.prune(Bq, F, R, forced=kept_gpu)
                if window is not None:
                    row_max[(bb, hh)] = rm[kept_gpu]
                    atol_rows = atol_rows[kept_gpu]
                if not do_check:
                    continue
                e = assert_scores_close(_unit_rows(cache.S[c], bb, hh, nk), o.S, rtol,
                                        "fused step %d S unit (%d,%d)" % (t, bb, hh),
                                        atol=atol_rows if atol_rows is not None else 0.0)
                rep.max_rel_err_decode = max(rep.max_rel_err_decode, e)
                assert_scores_close(_unit_rows(cache.nrm[c], bb, hh, nk), o.nrm, rtol, "fused nrm")
                assert np.array_equal(_unit_rows(cache.K[c], bb, hh, nk), o.K), "fused: K rows differ from oracle"
                assert np.array_equal(_unit_rows(cache.V[c], bb, hh, nk), o.V), "fused: V rows differ from oracle"
                assert np.array_equal(cache.pos[c][bb, hh, :nk].cpu().numpy(), o.pos), "fused: positions differ"

        for t in range(T if fused else 0):
            new_pos = [L + t for L in inp.lens]
            n_before = [n + 1 for n in cache.lens]
            cache.decode_prune_step(qd[t], kd[t], vd[t], new_pos)
            for (bb, hh), o in heads.items():
                o.append_and_score(q_of(inp.qd[t], bb, hh), _vec(inp.kd[t, bb, hh]), _vec(inp.vd[t, bb, hh]),
                                   new_pos[bb])
            check_fused_step(t, n_before, (t % check_every == 0) or t == T - 1)

        for t in range(0 if fused else T):
            c = cache.cur
            new_pos = [L + t for L in inp.lens]
            cache.decode_step(qd[t], kd[t], vd[t], new_pos)
            n_before = list(cache.lens)
            do_check = (t % check_every == 0) or t == T - 1
            if do_check:
                torch.cuda.synchronize()
            for (bb, hh), o in heads.items():
                o.append_and_score(q_of(inp.qd[t], bb, hh), _vec(inp.kd[t, bb, hh]), _vec(inp.vd[t, bb, hh]),
                                   new_pos[bb])
                if do_check:
                    n = n_before[bb]
                    e = assert_scores_close(_unit_rows(cache.S[c], bb, hh, n), o.S, rtol,
                                            "decode S step %d unit (%d,%d)" % (t, bb, hh))
                    rep.max_rel_err_decode = max(rep.max_rel_err_decode, e)
                    assert_scores_close(_unit_rows(cache.nrm[c], bb, hh, n), o.nrm, rtol, "decode nrm")
            cache.prune()
            check_prune(cache.K[c], cache.V[c], cache.S[c], cache.nrm[c], cache.pos[c], n_before)
        return rep
    finally:
        torch.cuda.synchronize()
        cache.close()
