"""Checks the oracle against the few numbers the paper itself prints (tests/golden)."""
import os
from fractions import Fraction

import numpy as np

from oracle import vatp_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _facts():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_facts.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [s.strip() for s in line.split("=")]
            out[k] = Fraction(v)
    return out


def test_norm_state_is_one_over_2d_of_the_kv_state():
    f = _facts()
    d = int(f["d_head_7b"])
    n = 37
    h = orc.OracleHead(d)
    rng = np.random.default_rng(0)
    h.prefill(rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d)))
    assert Fraction(h.nrm.size, h.K.size + h.V.size) == f["norm_state_over_kv_state"]


def test_paper_budget_split_keeps_exactly_the_budget():
    # LLaMA2 setting of the paper: prompt 4096, budget half of it, half of the budget a
    # local window, the first F tokens always kept (F counted inside the budget here).
    f = _facts()
    L = int(f["llama2_max_prompt"])
    B = int(L * f["budget_fraction_of_prompt"])
    R = int(B * (1 - f["h2o_importance_share_of_budget"]))
    F = int(f["forced_prefix_llama2"])
    I = np.random.default_rng(1).random(L)
    kept = orc.select(I, B, F, R)
    assert len(kept) == B == 2048
    assert kept[:F].tolist() == list(range(F)) and kept[-R:].tolist() == list(range(L - R, L))
    heavy = kept[F:-R]
    assert len(heavy) == B - F - R
    cand = I[F:L - R]
    assert np.sort(I[heavy])[0] >= np.sort(cand)[::-1][len(heavy) - 1]


def test_units_driver_equals_single_head_steps():
    import ctypes
    rng = np.random.default_rng(2)
    units, cap, d, F, R = 3, 16, 4, 1, 2
    n = np.array([16, 9, 12], dtype=np.int64)
    B = np.array([15, 9, 6], dtype=np.int64)
    K, V = rng.standard_normal((units, cap, d)), rng.standard_normal((units, cap, d))
    S = rng.random((units, cap))
    q = rng.standard_normal((units, d))
    nrm = np.abs(V).sum(-1)
    Ko, Vo, So, No = np.zeros_like(K), np.zeros_like(V), np.zeros_like(S), np.zeros_like(S)
    kept = np.zeros((units, cap), dtype=np.int32)
    n_out = np.zeros(units, dtype=np.int64)
    S_in = S.copy()
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    i64 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    orc.lib().vatp_oracle_decode_prune_units(
        p(q), p(K), p(V), p(S_in), p(nrm), units, cap, i64(n), d, 0.5, i64(B), F, R,
        p(Ko), p(Vo), p(So), p(No), kept.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), i64(n_out))
    for u in range(units):
        nu = int(n[u])
        S1, _ = orc.decode_scores(q[u], K[u, :nu], S[u, :nu], 0.5)
        k = orc.select(orc.importance(S1, nrm[u, :nu]), int(B[u]), F, R)
        assert n_out[u] == len(k)
        np.testing.assert_array_equal(kept[u, :len(k)], k)
        np.testing.assert_array_equal(Ko[u, :len(k)], K[u, k])
        np.testing.assert_array_equal(Vo[u, :len(k)], V[u, k])
        np.testing.assert_array_equal(So[u, :len(k)], S1[k])
        np.testing.assert_array_equal(No[u, :len(k)], nrm[u, k])
