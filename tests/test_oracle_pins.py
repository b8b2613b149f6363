"""Pins for the float64 CPU oracle: things the paper and the mathematics fix,
none of which re-use the oracle's own code.

  brute force      full attention matrix in pure Python (Eq. 1, 2, 4) on tiny inputs
  library routine  torch float64 softmax / abs-sum / stable sort
  closed forms     uniform attention -> harmonic sums (exact Fractions)
  invariants       softmax rows sum to one; kept count equals the budget; protected rows
  reductions       uniform value norms -> attention-only ranking; B = F + R -> sinks+window
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import bruteforce as bf
from oracle import vatp_oracle as orc


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("L,d,seed", [(1, 1, 0), (2, 3, 1), (7, 4, 2), (19, 8, 3), (32, 8, 4)])
def test_prefill_scores_match_bruteforce(L, d, seed):
    rng = np.random.default_rng(seed)
    Q, K = 2.0 * _rand(rng, L, d), 1.5 * _rand(rng, L, d)
    c = 1.0 / math.sqrt(d)
    A = bf.attention_matrix(Q.tolist(), K.tolist(), c)
    S_bf = bf.accumulated_scores(A)
    S = orc.prefill_scores(Q, K)
    np.testing.assert_allclose(S, S_bf, rtol=1e-12, atol=0)


def test_l1norm_and_importance_match_bruteforce():
    rng = np.random.default_rng(5)
    V = _rand(rng, 23, 8)
    S = rng.random(23)
    nrm = orc.l1norm(V)
    np.testing.assert_allclose(nrm, bf.l1(V.tolist()), rtol=1e-15)
    np.testing.assert_array_equal(orc.importance(S, nrm), S * nrm)


@pytest.mark.parametrize("n,B,F,R,seed", [(32, 16, 2, 4, 0), (32, 31, 0, 0, 1), (17, 9, 3, 6, 2),
                                          (20, 20, 2, 4, 3), (12, 30, 2, 4, 4), (25, 7, 0, 7, 5)])
def test_select_matches_sorted_bruteforce(n, B, F, R, seed):
    rng = np.random.default_rng(seed)
    I = rng.random(n)
    I[rng.integers(0, n, 6)] = 0.25          # planted exact ties
    kept = orc.select(I, B, F, R)
    assert kept.tolist() == bf.keep_set(I.tolist(), n, B, F, R)


@pytest.mark.parametrize("seed,B,F,R", [(0, 12, 2, 4), (1, 10, 0, 0), (2, 9, 1, 8)])
def test_decode_trajectory_matches_bruteforce_replay(seed, B, F, R):
    rng = np.random.default_rng(100 + seed)
    L, d, T = 24, 6, 10
    Q, K, V = _rand(rng, L, d) * 2, _rand(rng, L, d) * 2, _rand(rng, L, d)
    V *= np.exp(0.7 * _rand(rng, L, 1))
    qd, kd, vd = _rand(rng, T, d) * 2, _rand(rng, T, d) * 2, _rand(rng, T, d)
    c = 1.0 / math.sqrt(d)
    want = bf.replay(Q.tolist(), K.tolist(), V.tolist(), qd.tolist(), kd.tolist(), vd.tolist(),
                     c, B, F, R)
    h = orc.OracleHead(d)
    h.prefill(Q, K, V)
    kept = h.prune(B, F, R)
    got = [(h.pos.tolist(), h.S.copy(), kept.tolist())]
    for t in range(T):
        h.append_and_score(qd[t], kd[t], vd[t], L + t)
        kept = h.prune(B, F, R)
        got.append((h.pos.tolist(), h.S.copy(), kept.tolist()))
    assert len(got) == len(want)
    for (gp, gS, gk), (wp, wS, wk) in zip(got, want):
        assert gp == wp and gk == wk
        np.testing.assert_allclose(gS, wS, rtol=1e-12)


# ---------------------------------------------------------------- library routines

@pytest.mark.parametrize("L,d", [(257, 64), (1024, 128)])
def test_prefill_scores_match_torch_softmax(L, d):
    g = torch.Generator().manual_seed(L)
    Q = torch.randn(L, d, generator=g, dtype=torch.float64) * 1.3
    K = torch.randn(L, d, generator=g, dtype=torch.float64)
    logits = (Q @ K.T) / math.sqrt(d)
    logits = logits.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    want = torch.softmax(logits, dim=-1).sum(dim=0).numpy()
    got = orc.prefill_scores(Q.numpy(), K.numpy())
    np.testing.assert_allclose(got, want, rtol=1e-11)


def test_decode_scores_match_torch_softmax():
    g = torch.Generator().manual_seed(9)
    n, d = 333, 128
    K = torch.randn(n, d, generator=g, dtype=torch.float64)
    q = torch.randn(d, generator=g, dtype=torch.float64) * 2
    S0 = torch.rand(n, generator=g, dtype=torch.float64)
    a = torch.softmax(K @ q / math.sqrt(d), dim=0)
    S1, a_got = orc.decode_scores(q.numpy(), K.numpy(), S0.numpy())
    np.testing.assert_allclose(a_got, a.numpy(), rtol=1e-12)
    np.testing.assert_allclose(S1, (S0 + a).numpy(), rtol=1e-13)


def test_l1norm_matches_torch():
    g = torch.Generator().manual_seed(3)
    V = torch.randn(100, 128, generator=g, dtype=torch.float64)
    np.testing.assert_allclose(orc.l1norm(V.numpy()), V.abs().sum(-1).numpy(), rtol=1e-14)


def test_select_matches_stable_argsort():
    rng = np.random.default_rng(11)
    n, B, F, R = 3000, 900, 20, 100
    I = np.round(rng.random(n), 3)            # many exact ties
    order = np.argsort(-I[F:n - R], kind="stable") + F
    want = np.sort(np.concatenate([np.arange(F), order[:B - F - R], np.arange(n - R, n)]))
    np.testing.assert_array_equal(orc.select(I, B, F, R), want)


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("L", [1, 5, 64])
def test_uniform_attention_gives_harmonic_sums(L):
    d = 4
    K = np.random.default_rng(L).standard_normal((L, d))
    Q = np.zeros((L, d))
    want = [float(x) for x in bf.harmonic_scores(L)]
    np.testing.assert_allclose(orc.prefill_scores(Q, K), want, rtol=1e-13)
    # equal keys give the same uniform attention, whatever the queries are
    Q2 = np.random.default_rng(L + 1).standard_normal((L, d))
    np.testing.assert_allclose(orc.prefill_scores(Q2, np.tile(K[:1], (L, 1))), want, rtol=1e-12)


def test_uniform_attention_equal_norms_keeps_oldest_candidates():
    L, d, B, F, R = 40, 4, 20, 3, 5
    S = orc.prefill_scores(np.zeros((L, d)), np.ones((L, d)))
    assert np.all(np.diff(S) < 0)                       # H_L - H_i strictly decreasing
    kept = orc.select(orc.importance(S, np.full(L, 7.0)), B, F, R)
    assert kept.tolist() == list(range(B - R)) + list(range(L - R, L))


def test_group_onehot_attention_gives_per_group_harmonic_sums():
    # tokens alternate between two groups; a very large logit inside the own group makes
    # attention uniform over the earlier tokens of the same group
    L, beta = 12, 60.0
    grp = [j % 2 for j in range(L)]
    E = np.eye(2)
    Q = np.array([beta * E[g] for g in grp])
    K = np.array([beta * E[g] for g in grp])
    S = orc.prefill_scores(Q, K, c=1.0)
    for i in range(L):
        same = [j for j in range(L) if grp[j] == grp[i]]
        rank = {j: r for r, j in enumerate(same)}
        want = sum(Fraction(1, rank[j] + 1) for j in same if j >= i)
        assert S[i] == pytest.approx(float(want), rel=1e-12)


# ---------------------------------------------------------------- invariants

def test_softmax_rows_sum_to_one_invariants():
    rng = np.random.default_rng(21)
    L, d = 300, 16
    Q, K = 3 * _rand(rng, L, d), 3 * _rand(rng, L, d)
    S = orc.prefill_scores(Q, K)
    assert S.sum() == pytest.approx(L, rel=1e-12)       # every query row distributes mass 1
    assert S[0] >= 1.0                                  # a_0^0 = 1
    assert 0.0 < S[-1] <= 1.0                           # only the last query sees the last key
    assert np.all(S > 0)
    q = _rand(rng, d)
    S2, a = orc.decode_scores(q, K, S)
    assert a.sum() == pytest.approx(1.0, rel=1e-13)
    assert S2.sum() == pytest.approx(L + 1.0, rel=1e-12)


def test_key_shift_leaves_scores_unchanged_and_value_scale_is_homogeneous():
    rng = np.random.default_rng(22)
    L, d = 64, 8
    Q, K, V = _rand(rng, L, d), _rand(rng, L, d), _rand(rng, L, d)
    S = orc.prefill_scores(Q, K)
    np.testing.assert_allclose(orc.prefill_scores(Q, K + _rand(rng, 1, d)), S, rtol=1e-10)
    alpha = rng.random(L) + 0.5
    I = orc.importance(S, orc.l1norm(V))
    I2 = orc.importance(S, orc.l1norm(V * alpha[:, None]))
    np.testing.assert_allclose(I2, alpha * I, rtol=1e-13)
    assert orc.select(I, 20, 2, 4).tolist() == orc.select(8.0 * I, 20, 2, 4).tolist()
    # swapping Q and K is a different computation: a transposed operand cannot pass unnoticed
    assert not np.allclose(orc.prefill_scores(K, Q), S, rtol=1e-3)


@pytest.mark.parametrize("n,B,F,R", [(100, 40, 2, 8), (100, 99, 0, 0), (50, 10, 5, 5), (9, 9, 1, 1)])
def test_selection_invariants(n, B, F, R):
    rng = np.random.default_rng(n + B)
    I = rng.random(n)
    kept = orc.select(I, B, F, R)
    assert len(kept) == min(n, B)
    assert np.all(np.diff(kept) > 0)
    assert set(range(F)) <= set(kept.tolist())
    assert set(range(n - R, n)) <= set(kept.tolist())
    dropped = sorted(set(range(n)) - set(kept.tolist()))
    heavy = [r for r in kept.tolist() if F <= r < n - R]
    if dropped and heavy:
        assert min(I[heavy]) >= max(I[dropped])
    rows = rng.standard_normal((n, 5))
    np.testing.assert_array_equal(orc.gather_rows(rows, kept), rows[kept])   # bit-for-bit


def test_budget_smaller_than_protected_rows_is_an_error():
    with pytest.raises(ValueError):
        orc.select(np.ones(50), 9, 4, 6)


# ---------------------------------------------------------------- reductions to known methods

def test_uniform_value_norms_reduce_to_attention_only_ranking():
    rng = np.random.default_rng(31)
    L, d, B, F, R = 200, 16, 60, 2, 10
    Q, K = 2 * _rand(rng, L, d), 2 * _rand(rng, L, d)
    V = rng.choice([-1.0, 1.0], size=(L, d))            # every row has l1 norm exactly d
    S = orc.prefill_scores(Q, K)
    nrm = orc.l1norm(V)
    assert np.all(nrm == d)
    vatp = orc.select(orc.importance(S, nrm), B, F, R)
    attn_only = orc.select(S, B, F, R)
    assert vatp.tolist() == attn_only.tolist()
    # and a non-uniform norm does change the set (the metric is not attention-only)
    nrm2 = nrm * np.exp(rng.standard_normal(L))
    assert orc.select(orc.importance(S, nrm2), B, F, R).tolist() != attn_only.tolist()


def test_zero_importance_slots_reduce_to_sinks_plus_window():
    rng = np.random.default_rng(32)
    n, F, R = 80, 4, 12
    kept = orc.select(rng.random(n), F + R, F, R)
    assert kept.tolist() == list(range(F)) + list(range(n - R, n))


def test_exact_ties_keep_lowest_indices_and_evict_one_takes_last_minimum():
    n, F, R = 30, 2, 4
    I = np.linspace(1.0, 2.0, n)
    zero_rows = [5, 9, 10, 17, 21]
    I[zero_rows] = 0.0                                  # e.g. all-zero value rows
    kept = orc.select(I, n - 2, F, R)                   # evict two of the five tied rows
    assert sorted(set(range(n)) - set(kept.tolist())) == [17, 21]
    I2 = np.array([3.0, 1.0, 2.0, 1.0, 5.0, 1.0, 4.0])
    kept = orc.select(I2, len(I2) - 1, 0, 0)            # F = R = 0, evict one
    assert sorted(set(range(7)) - set(kept.tolist())) == [5]


def test_splitting_units_gives_identical_results():
    rng = np.random.default_rng(33)
    units, cap, d = 3, 20, 4
    lens = np.array([20, 7, 13], dtype=np.int64)
    Q, K = _rand(rng, units, cap, d), _rand(rng, units, cap, d)
    S = np.zeros((units, cap))
    import ctypes
    f64p = ctypes.POINTER(ctypes.c_double)
    orc.lib().vatp_oracle_prefill_scores_units(
        Q.ctypes.data_as(f64p), K.ctypes.data_as(f64p), units, cap,
        lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), d, 0.5, S.ctypes.data_as(f64p))
    for u in range(units):
        np.testing.assert_array_equal(S[u, :lens[u]], orc.prefill_scores(Q[u, :lens[u]], K[u, :lens[u]], 0.5))


def test_tail_scores_equal_the_tail_of_the_full_pass():
    rng = np.random.default_rng(34)
    L, d = 90, 8
    Q, K = _rand(rng, L, d), _rand(rng, L, d)
    full = orc.prefill_scores(Q, K)
    np.testing.assert_allclose(orc.prefill_scores_tail(Q, K, 60), full[60:], rtol=1e-13)
    np.testing.assert_array_equal(orc.prefill_scores_tail(Q, K, 0), full)
    np.testing.assert_array_equal(orc.prefill_scores_units(Q[None], K[None], [L])[0], full)


# ---------------------------------------------------------------- norm ablation (Table 2)

def test_value_norms_match_numpy_and_their_inequalities():
    rng = np.random.default_rng(41)
    V = _rand(rng, 50, 16) * np.exp(_rand(rng, 50, 1))
    n1, n2, ninf = orc.vnorm(V, 0), orc.vnorm(V, 1), orc.vnorm(V, 2)
    np.testing.assert_array_equal(n1, orc.l1norm(V))
    np.testing.assert_allclose(n1, np.linalg.norm(V, 1, axis=1), rtol=1e-14)
    np.testing.assert_allclose(n2, np.linalg.norm(V, 2, axis=1), rtol=1e-14)
    np.testing.assert_allclose(ninf, np.linalg.norm(V, np.inf, axis=1), rtol=0)
    assert np.all(ninf <= n2 * (1 + 1e-15)) and np.all(n2 <= n1 * (1 + 1e-15)) and np.all(n1 <= 4.0 * n2 * (1 + 1e-15))
    onehot = np.eye(16)[[3, 7]] * np.array([[2.5], [-4.0]])
    for kind in (0, 1, 2):
        np.testing.assert_array_equal(orc.vnorm(onehot, kind), [2.5, 4.0])      # all three agree on one-hot rows
    # kind 3 switches the norm off: the ranking is then the accumulated attention score alone
    np.testing.assert_array_equal(orc.vnorm(V, 3), np.ones(50))
    S = rng.random(50) + 0.1
    np.testing.assert_array_equal(orc.select(orc.importance(S, orc.vnorm(V, 3)), 20, 2, 5), orc.select(S, 20, 2, 5))


def test_norm_choice_changes_the_kept_set_only_through_the_norm():
    rng = np.random.default_rng(42)
    L, d, B, F, R = 120, 8, 40, 2, 8
    Q, K, V = _rand(rng, L, d) * 2, _rand(rng, L, d) * 2, _rand(rng, L, d) * np.exp(_rand(rng, L, 1))
    sets = []
    for kind in (0, 1, 2):
        h = orc.OracleHead(d, norm_kind=kind)
        h.prefill(Q, K, V)
        np.testing.assert_array_equal(h.nrm, orc.vnorm(V, kind))
        kept = h.prune(B, F, R)
        assert kept.tolist() == orc.select(orc.importance(orc.prefill_scores(Q, K), orc.vnorm(V, kind)), B, F, R).tolist()
        sets.append(kept.tolist())
    assert sets[0] != sets[2]                       # l1 and l-infinity rank differently on this data


# ---------------------------------------------------------------- scores from given row normalisers

def test_row_lse_matches_torch_logsumexp_and_closes_the_loop():
    g = torch.Generator().manual_seed(51)
    L, d = 150, 16
    Q = torch.randn(L, d, generator=g, dtype=torch.float64) * 1.7
    K = torch.randn(L, d, generator=g, dtype=torch.float64)
    logits = (Q @ K.T) / math.sqrt(d)
    logits = logits.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    lse = orc.row_lse(Q.numpy(), K.numpy())
    np.testing.assert_allclose(lse, torch.logsumexp(logits, dim=-1).numpy(), rtol=1e-13)
    S = orc.prefill_scores_given_lse(Q.numpy(), K.numpy(), lse)
    np.testing.assert_allclose(S, orc.prefill_scores(Q.numpy(), K.numpy()), rtol=1e-12)
    np.testing.assert_allclose(S, torch.exp(logits - torch.from_numpy(lse)[:, None]).sum(0).numpy(), rtol=1e-12)
    # a shifted normaliser scales every weight of that row: S is linear in exp(-lse)
    S2 = orc.prefill_scores_given_lse(Q.numpy(), K.numpy(), lse + math.log(2.0))
    np.testing.assert_allclose(S2, S / 2.0, rtol=1e-12)


# ---------------------------------------------------------------- attention output (Eq. 1)

def test_attention_output_matches_torch_and_simple_cases():
    g = torch.Generator().manual_seed(61)
    n, d = 77, 16
    K = torch.randn(n, d, generator=g, dtype=torch.float64)
    V = torch.randn(n, d, generator=g, dtype=torch.float64)
    q = torch.randn(d, generator=g, dtype=torch.float64) * 2
    a = torch.softmax(K @ q / math.sqrt(d), dim=0)
    out, abs_out = orc.attention_output(q.numpy(), K.numpy(), V.numpy())
    np.testing.assert_allclose(out, (a[:, None] * V).sum(0).numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(abs_out, (a[:, None] * V.abs()).sum(0).numpy(), rtol=1e-12)
    # uniform attention (q = 0) averages the value rows; one row returns that row
    out0, _ = orc.attention_output(np.zeros(d), K.numpy(), V.numpy())
    np.testing.assert_allclose(out0, V.mean(0).numpy(), rtol=1e-12, atol=1e-15)
    out1, _ = orc.attention_output(q.numpy(), K[:1].numpy(), V[:1].numpy())
    np.testing.assert_array_equal(out1, V[0].numpy())
    # the weights are those of the decode score update
    _, a_dec = orc.decode_scores(q.numpy(), K.numpy(), np.zeros(n))
    np.testing.assert_allclose(out, a_dec @ V.numpy(), rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- history-window scores (Eq. 3)

@pytest.mark.parametrize("L,d,w", [(1, 4, 0), (7, 4, 0), (9, 8, 3), (20, 8, 5), (20, 8, 19), (20, 8, 50), (31, 16, 10)])
def test_window_scores_match_bruteforce(L, d, w):
    rng = np.random.default_rng(100 + L + w)
    Q, K = _rand(rng, L, d) * 1.5, _rand(rng, L, d) * 1.5
    c = orc.default_scale(d)
    A = bf.attention_matrix(Q.tolist(), K.tolist(), c)
    S, P = orc.prefill_window(Q, K, w)
    np.testing.assert_allclose(S, bf.windowed_scores(A, w, L - 1), rtol=1e-13, atol=1e-300)
    j0 = max(0, L - 1 - w)
    assert P.shape == (L - j0, L)
    np.testing.assert_allclose(P, np.array(A)[j0:], rtol=1e-13, atol=0)


def test_window_scores_special_cases():
    rng = np.random.default_rng(7)
    L, d = 40, 8
    Q, K = _rand(rng, L, d), _rand(rng, L, d)
    # a window that covers the whole prompt is the accumulated score (Eq. 2)
    for w in (L - 1, L, 10 * L):
        np.testing.assert_allclose(orc.prefill_window(Q, K, w)[0], orc.prefill_scores(Q, K), rtol=1e-14)
    # w = 0: only the last query's attention row
    S0, P0 = orc.prefill_window(Q, K, 0)
    want = torch.softmax(torch.from_numpy(Q[-1] @ K.T * orc.default_scale(d)), dim=0).numpy()
    np.testing.assert_allclose(S0, want, rtol=1e-13)
    assert P0.shape == (1, L)
    # every attention row sums to one: the scores total the number of rows in the window
    for w in (0, 3, 17, 39, 100):
        S, P = orc.prefill_window(Q, K, w)
        assert abs(S.sum() - min(L, w + 1)) < 1e-12
        np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=1e-13)
        assert np.all(np.triu(P, k=L - P.shape[0] + 1) == 0.0)      # causal: nothing right of the diagonal
    # a longer window never lowers a score
    assert np.all(orc.prefill_window(Q, K, 9)[0] >= orc.prefill_window(Q, K, 5)[0] - 1e-15)


def test_window_scores_uniform_attention_closed_form():
    """Identical keys give a_k^j = 1/(j+1): S_k = sum_{j=max(L-1-w,k)}^{L-1} 1/(j+1), exactly."""
    L, d, w = 25, 4, 6
    Q = _rand(np.random.default_rng(3), L, d)
    K = np.tile(np.array([[0.3, -0.2, 0.5, 0.1]]), (L, 1))
    S, _ = orc.prefill_window(Q, K, w)
    want = [float(sum(Fraction(1, j + 1) for j in range(max(L - 1 - w, k), L))) for k in range(L)]
    np.testing.assert_allclose(S, want, rtol=1e-14)


def test_window_head_replay_matches_literal_equation_without_pruning():
    """Prompt + decode steps with a budget that never prunes: after every step the head's scores are
    Eq. 3 read off the full attention matrix of the whole sequence so far."""
    rng = np.random.default_rng(11)
    L, T, d, w = 12, 9, 4, 5
    Q, K, V = _rand(rng, L + T, d) * 1.3, _rand(rng, L + T, d) * 1.3, _rand(rng, L + T, d)
    c = orc.default_scale(d)
    A = bf.attention_matrix(Q.tolist(), K.tolist(), c)
    h = orc.OracleHead(d, window=w)
    h.prefill(Q[:L], K[:L], V[:L])
    np.testing.assert_allclose(h.S, bf.windowed_scores(A, w, L - 1), rtol=1e-13)
    for t in range(L, L + T):
        h.append_and_score(Q[t], K[t], V[t], t)
        np.testing.assert_allclose(h.S, bf.windowed_scores(A, w, t), rtol=1e-12, atol=1e-300)
        assert len(h.hist) == min(t + 1, w + 1)


def test_window_head_with_pruning_keeps_history_aligned():
    """With pruning: the history columns follow the kept rows, a token's score is the sum of what it
    received in the last w+1 steps, and a token nobody attends to for w+1 steps drops to the tiny
    weights it actually got."""
    rng = np.random.default_rng(12)
    L, T, d, w, B, F, R = 30, 14, 8, 4, 16, 2, 3
    Q, K, V = _rand(rng, L + T, d) * 1.5, _rand(rng, L + T, d) * 1.5, _rand(rng, L + T, d) * np.exp(_rand(rng, L + T, 1))
    h = orc.OracleHead(d, window=w)
    h.prefill(Q[:L], K[:L], V[:L])
    kept = h.prune(B, F, R)
    assert len(kept) == B and all(row.shape == (B,) for row in h.hist)
    received = {int(p): [] for p in h.pos}          # per surviving token: attention received per decode step
    for t in range(L, L + T):
        a = h.append_and_score(Q[t], K[t], V[t], t)
        for p, ai in zip(h.pos, a):
            received.setdefault(int(p), []).append(ai)
        assert abs(a.sum() - 1.0) < 1e-12
        assert h.S.sum() <= w + 1 + 1e-12 and np.all(h.S >= 0)
        h.prune(B, F, R)
        assert all(row.shape == (h.n,) for row in h.hist)
        if t - L + 1 >= w + 1:                      # the prompt's rows have left the window
            for p, s in zip(h.pos, h.S):
                np.testing.assert_allclose(s, sum(received[int(p)][-(w + 1):]), rtol=1e-12, atol=1e-300)


# ---------------------------------------------------------------- grouped-query attention

@pytest.mark.parametrize("g,seed,B,F,R", [(2, 0, 12, 2, 4), (3, 1, 10, 0, 0), (8, 2, 9, 1, 6)])
def test_group_trajectory_matches_bruteforce_replay(g, seed, B, F, R):
    rng = np.random.default_rng(300 + seed)
    L, d, T = 22, 6, 9
    Qg, K, V = _rand(rng, g, L, d) * 2, _rand(rng, L, d) * 2, _rand(rng, L, d) * np.exp(0.7 * _rand(rng, L, 1))
    qdg, kd, vd = _rand(rng, T, g, d) * 2, _rand(rng, T, d) * 2, _rand(rng, T, d)
    c = 1.0 / math.sqrt(d)
    want = bf.replay_group(Qg.tolist(), K.tolist(), V.tolist(), qdg.tolist(), kd.tolist(), vd.tolist(), c, B, F, R)
    h = orc.OracleHead(d, group=g)
    h.prefill(Qg, K, V)
    kept = h.prune(B, F, R)
    got = [(h.pos.tolist(), h.S.copy(), kept.tolist())]
    for t in range(T):
        a = h.append_and_score(qdg[t], kd[t], vd[t], L + t)
        assert abs(a.sum() - 1.0) < 1e-14           # a mean of g softmax rows still sums to one
        kept = h.prune(B, F, R)
        got.append((h.pos.tolist(), h.S.copy(), kept.tolist()))
    assert len(got) == len(want)
    for (gp, gS, gk), (wp, wS, wk) in zip(got, want):
        assert gp == wp and gk == wk
        np.testing.assert_allclose(gS, wS, rtol=1e-12)


def test_group_scores_match_torch_softmax_mean():
    gen = torch.Generator().manual_seed(77)
    g, L, d = 4, 193, 64
    Q = torch.randn(g, L, d, generator=gen, dtype=torch.float64) * 1.3
    K = torch.randn(L, d, generator=gen, dtype=torch.float64)
    logits = torch.einsum("gjd,id->gji", Q, K) / math.sqrt(d)
    logits = logits.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    want = torch.softmax(logits, dim=-1).sum(dim=1).mean(dim=0).numpy()
    got = orc.prefill_scores_group(Q.numpy(), K.numpy())
    np.testing.assert_allclose(got, want, rtol=1e-11)
    assert abs(got.sum() - L) < 1e-9
    # decode step: mean of the heads' softmax rows
    q = torch.randn(g, d, generator=gen, dtype=torch.float64) * 2
    S0 = torch.rand(L, generator=gen, dtype=torch.float64)
    a = torch.softmax(q @ K.T / math.sqrt(d), dim=-1).mean(dim=0)
    S1, a_got = orc.decode_scores_group(q.numpy(), K.numpy(), S0.numpy())
    np.testing.assert_allclose(a_got, a.numpy(), rtol=1e-12)
    np.testing.assert_allclose(S1, (S0 + a).numpy(), rtol=1e-13)


def test_group_of_one_and_group_of_equal_heads_reduce_to_a_single_head():
    rng = np.random.default_rng(31)
    L, d = 40, 8
    Q, K = _rand(rng, L, d) * 1.5, _rand(rng, L, d)
    S1 = orc.prefill_scores(Q, K)
    np.testing.assert_array_equal(orc.prefill_scores_group(Q[None], K), S1)
    np.testing.assert_array_equal(orc.prefill_scores_group(np.stack([Q] * 4), K), S1)     # (4x)/4 is exact
    np.testing.assert_allclose(orc.prefill_scores_group(np.stack([Q] * 3), K), S1, rtol=1e-15)
    # the many-heads form is the same function, unit by unit (ragged lengths included)
    Qg = _rand(rng, 3, 2, L, d)
    Ku = _rand(rng, 3, L, d)
    lens = [L, 17, 1]
    many = orc.prefill_scores_group_units(Qg, Ku, lens)
    for u, n in enumerate(lens):
        np.testing.assert_array_equal(many[u, :n], orc.prefill_scores_group(Qg[u, :, :n], Ku[u, :n]))


def test_group_mean_is_taken_after_each_heads_softmax():
    """Two heads whose scores are known in closed form: head A has zero queries (uniform attention,
    harmonic sums), head B puts all its attention on key 0.  The group score is the mean of the two;
    a sum, a softmax over mean logits or a softmax over both heads' logits together would all differ."""
    L, d, beta = 12, 4, 60.0
    K = np.zeros((L, d))
    K[0, 0] = beta                       # only key 0 has a component along e_0
    K[1:, 1] = 1.0
    QA = np.zeros((L, d))
    QB = np.zeros((L, d))
    QB[:, 0] = beta                      # logit of key 0: c * beta^2 = 1800, every other logit 0
    S = orc.prefill_scores_group(np.stack([QA, QB]), K)
    harm = np.array([float(x) for x in bf.harmonic_scores(L)])
    sB = np.zeros(L)
    sB[0] = L                            # exp(-1800) underflows to 0: the rest receives nothing
    np.testing.assert_allclose(S, (harm + sB) / 2, rtol=1e-14)
    # the attention-only ranking of the group therefore starts with token 0, then the oldest tokens
    kept = orc.select(S, 5, 0, 0)
    assert kept.tolist() == [0, 1, 2, 3, 4]


def test_group_window_replay_matches_literal_equation_without_pruning():
    """Grouped queries with a history window: after the prompt and after every decode step (no pruning) the
    scores are Eq. 3 read off the g full attention matrices, averaged over the group."""
    rng = np.random.default_rng(41)
    g, L, T, d, w = 3, 11, 8, 4, 4
    Qg, K, V = _rand(rng, g, L + T, d) * 1.3, _rand(rng, L + T, d) * 1.3, _rand(rng, L + T, d)
    c = orc.default_scale(d)
    A = [bf.attention_matrix(Qg[r].tolist(), K.tolist(), c) for r in range(g)]
    want = lambda t: bf.group_mean([bf.windowed_scores(A[r], w, t) for r in range(g)])
    h = orc.OracleHead(d, window=w, group=g)
    h.prefill(Qg[:, :L], K[:L], V[:L])
    np.testing.assert_allclose(h.S, want(L - 1), rtol=1e-13)
    assert len(h.hist) == min(L, w + 1)
    for t in range(L, L + T):
        h.append_and_score(Qg[:, t], K[t], V[t], t)
        np.testing.assert_allclose(h.S, want(t), rtol=1e-12, atol=1e-300)
    # one head in the group, or a window that covers everything, reduce to what is pinned elsewhere
    S1, P1 = orc.prefill_window_group(Qg[:1, :L], K[:L], w)
    S0, P0 = orc.prefill_window(Qg[0, :L], K[:L], w)
    np.testing.assert_array_equal(S1, S0)
    np.testing.assert_array_equal(P1, P0)
    Sall, _ = orc.prefill_window_group(Qg[:, :L], K[:L], L)
    np.testing.assert_allclose(Sall, orc.prefill_scores_group(Qg[:, :L], K[:L]), rtol=1e-14)
