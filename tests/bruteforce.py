"""Literal, pure-Python restatement of the paper's equations for tiny inputs.

Used only to pin the C oracle: it materialises the whole causal attention matrix
(Eq. 1), sums its columns (Eq. 2; over a history window, Eq. 3), multiplies by the value l1 norm (Eq. 4) and sorts.
No numpy arithmetic, no blocking; lists of Python floats (binary64) or Fractions.
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import List, Sequence


def attention_matrix(Q: Sequence[Sequence[float]], K: Sequence[Sequence[float]], c: float):
    """A[j][i] = a_i^j for i <= j, 0 above the diagonal."""
    L = len(Q)
    A = [[0.0] * L for _ in range(L)]
    for j in range(L):
        logits = [c * math.fsum(Q[j][x] * K[i][x] for x in range(len(Q[j]))) for i in range(j + 1)]
        m = max(logits)
        e = [math.exp(s - m) for s in logits]
        z = math.fsum(e)
        for i in range(j + 1):
            A[j][i] = e[i] / z
    return A


def accumulated_scores(A) -> List[float]:
    L = len(A)
    return [math.fsum(A[j][i] for j in range(i, L)) for i in range(L)]


def windowed_scores(A, w: int, t: int) -> List[float]:
    """Eq. 3 read literally off the full attention matrix: S_k^t = sum_{max(t-w,k) <= j <= t} a_k^j, k <= t."""
    return [math.fsum(A[j][k] for j in range(max(t - w, k), t + 1)) for k in range(t + 1)]


def l1(V) -> List[float]:
    return [math.fsum(abs(x) for x in row) for row in V]


def keep_set(I: Sequence[float], n: int, B: int, F: int, R: int) -> List[int]:
    if n <= B:
        return list(range(n))
    cand = list(range(F, n - R))
    ranked = sorted(cand, key=lambda r: (-I[r], r))
    heavy = ranked[: B - F - R]
    return sorted(set(range(F)) | set(heavy) | set(range(n - R, n)))


def harmonic_scores(L: int) -> List[Fraction]:
    """Uniform causal attention a_i^j = 1/(j+1)  =>  S_i = sum_{j=i}^{L-1} 1/(j+1)."""
    return [sum(Fraction(1, j + 1) for j in range(i, L)) for i in range(L)]


def replay(Q, K, V, qd, kd, vd, c, B, F, R):
    """Prompt pass + prune, then decode steps, rebuilding the row lists literally.
    Returns a list of (kept_positions, S_after_prune) per prune event."""
    L = len(Q)
    A = attention_matrix(Q, K, c)
    S = accumulated_scores(A)
    rows = [dict(k=list(K[i]), v=list(V[i]), S=S[i], pos=i) for i in range(L)]
    out = []

    def prune():
        nonlocal rows
        nrm = l1([r["v"] for r in rows])
        I = [rows[i]["S"] * nrm[i] for i in range(len(rows))]
        keep = keep_set(I, len(rows), B, F, R)
        rows = [rows[i] for i in keep]
        out.append(([r["pos"] for r in rows], [r["S"] for r in rows], keep))

    prune()
    for t in range(len(qd)):
        rows.append(dict(k=list(kd[t]), v=list(vd[t]), S=0.0, pos=L + t))
        logits = [c * math.fsum(qd[t][x] * r["k"][x] for x in range(len(qd[t]))) for r in rows]
        m = max(logits)
        e = [math.exp(s - m) for s in logits]
        z = math.fsum(e)
        for r, ei in zip(rows, e):
            r["S"] += ei / z
        prune()
    return out


def group_mean(rows: Sequence[Sequence[float]]) -> List[float]:
    """Element-wise mean of g equally long lists."""
    g = len(rows)
    return [math.fsum(row[i] for row in rows) / g for i in range(len(rows[0]))]


def replay_group(Qg, K, V, qdg, kd, vd, c, B, F, R):
    """`replay` for grouped-query attention: g query heads (Qg[r] prompt queries, qdg[t][r] the decode
    query of head r at step t) share the K/V rows; each head has its own softmax, the token score is
    the mean over the group of what the heads give it (Limitations section, paragraph on GQA)."""
    g, L = len(Qg), len(K)
    S = group_mean([accumulated_scores(attention_matrix(Qg[r], K, c)) for r in range(g)])
    rows = [dict(k=list(K[i]), v=list(V[i]), S=S[i], pos=i) for i in range(L)]
    out = []

    def prune():
        nonlocal rows
        nrm = l1([r["v"] for r in rows])
        I = [rows[i]["S"] * nrm[i] for i in range(len(rows))]
        keep = keep_set(I, len(rows), B, F, R)
        rows = [rows[i] for i in keep]
        out.append(([r["pos"] for r in rows], [r["S"] for r in rows], keep))

    prune()
    for t in range(len(qdg)):
        rows.append(dict(k=list(kd[t]), v=list(vd[t]), S=0.0, pos=L + t))
        weights = []
        for r in range(g):
            q = qdg[t][r]
            logits = [c * math.fsum(q[x] * row["k"][x] for x in range(len(q))) for row in rows]
            m = max(logits)
            e = [math.exp(s - m) for s in logits]
            z = math.fsum(e)
            weights.append([ei / z for ei in e])
        for row, a in zip(rows, group_mean(weights)):
            row["S"] += a
        prune()
    return out
