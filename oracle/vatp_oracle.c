/*
 * VATP reference oracle -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, float64 CPU statement of what the value-aware token pruning hot
 * path computes, written from the paper's equations.  It shares no code with the
 * HIP library; only tests, the smoke check and the CPU-baseline leg of the bench
 * may link or call it.
 *
 * Every function handles ONE attention head of ONE sequence ("each token in an
 * attention head" is scored on its own -- Methodology section, value-aware
 * pruning metric paragraph); the *_units drivers at the end only loop those
 * single-head functions over independent (sequence, head) units.
 *
 * Arrays are dense row-major doubles; a "row" is one token's d-vector.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/*
 * Accumulated attention score after a causal prompt pass (Eq. 2 with t = L-1,
 * attention weights a_i^j of Eq. 1 taken as softmax over the keys i <= j of the
 * scaled dot products c * <q_j, k_i>):
 *     S_i = sum_{j=i}^{L-1} a_i^j .
 * Q, K: [L, d].  S: [L] (overwritten).  scratch: [L] doubles.
 * j_start > 0 restricts the sum to query rows j >= j_start: the entries i >= j_start are
 * then still the complete S_i (no earlier query sees those keys), which lets a test check
 * the tail of a very long prompt without paying for all of its rows.
 */
void vatp_oracle_prefill_scores_from(const double *Q, const double *K, int64_t L, int64_t d,
                                     double c, int64_t j_start, double *S, double *scratch)
{
    for (int64_t i = 0; i < L; ++i) S[i] = 0.0;
    for (int64_t j = j_start; j < L; ++j) {
        const double *q = Q + j * d;
        double m = -INFINITY;
        for (int64_t i = 0; i <= j; ++i) {
            const double *k = K + i * d;
            double dot = 0.0;
            for (int64_t x = 0; x < d; ++x) dot += q[x] * k[x];
            scratch[i] = c * dot;
            if (scratch[i] > m) m = scratch[i];
        }
        double denom = 0.0;
        for (int64_t i = 0; i <= j; ++i) {
            scratch[i] = exp(scratch[i] - m);
            denom += scratch[i];
        }
        for (int64_t i = 0; i <= j; ++i) S[i] += scratch[i] / denom;
    }
}

void vatp_oracle_prefill_scores(const double *Q, const double *K, int64_t L, int64_t d,
                                double c, double *S, double *scratch)
{
    vatp_oracle_prefill_scores_from(Q, K, L, d, c, 0, S, scratch);
}

/*
 * Row log-sum-exp of the causal softmax of Eq. 1, natural logarithm:
 *     lse_j = ln sum_{i<=j} exp(c <q_j, k_i>),
 * the by-product a fused attention kernel hands back.  Q, K: [L, d] -> lse: [L].
 */
void vatp_oracle_row_lse(const double *Q, const double *K, int64_t L, int64_t d, double c,
                         double *lse, double *scratch)
{
    for (int64_t j = 0; j < L; ++j) {
        double m = -INFINITY;
        for (int64_t i = 0; i <= j; ++i) {
            double dot = 0.0;
            for (int64_t x = 0; x < d; ++x) dot += Q[j * d + x] * K[i * d + x];
            scratch[i] = c * dot;
            if (scratch[i] > m) m = scratch[i];
        }
        double denom = 0.0;
        for (int64_t i = 0; i <= j; ++i) denom += exp(scratch[i] - m);
        lse[j] = m + log(denom);
    }
}

/*
 * Eq. 2 after the prompt when the normalisers are given:  a_i^j = exp(c <q_j,k_i> - lse_j),
 *     S_i = sum_{j=i}^{L-1} a_i^j .
 */
void vatp_oracle_prefill_scores_given_lse(const double *Q, const double *K, const double *lse,
                                          int64_t L, int64_t d, double c, double *S)
{
    for (int64_t i = 0; i < L; ++i) {
        double s = 0.0;
        for (int64_t j = i; j < L; ++j) {
            double dot = 0.0;
            for (int64_t x = 0; x < d; ++x) dot += Q[j * d + x] * K[i * d + x];
            s += exp(c * dot - lse[j]);
        }
        S[i] = s;
    }
}

/*
 * One decode step of Eq. 2: the new query attends over all n rows currently in the
 * cache (the row of the new token included), and every row's accumulated score
 * grows by the attention weight it received:  S_r += a_r.
 * q: [d].  K: [n, d].  S: [n] in/out (the new row enters with S = 0).  a_out: [n] or NULL.
 */
void vatp_oracle_decode_scores(const double *q, const double *K, int64_t n, int64_t d,
                               double c, double *S, double *a_out, double *scratch)
{
    double m = -INFINITY;
    for (int64_t r = 0; r < n; ++r) {
        const double *k = K + r * d;
        double dot = 0.0;
        for (int64_t x = 0; x < d; ++x) dot += q[x] * k[x];
        scratch[r] = c * dot;
        if (scratch[r] > m) m = scratch[r];
    }
    double denom = 0.0;
    for (int64_t r = 0; r < n; ++r) {
        scratch[r] = exp(scratch[r] - m);
        denom += scratch[r];
    }
    for (int64_t r = 0; r < n; ++r) {
        double a = scratch[r] / denom;
        S[r] += a;
        if (a_out) a_out[r] = a;
    }
}

/*
 * Attention output of one query over a cache of n rows (Eq. 1):
 *     out[x] = sum_r a_r V[r][x],   a = softmax_r(c <q, K_r>).
 * q: [d].  K, V: [n, d].  out: [d].  abs_out (may be NULL): sum_r a_r |V[r][x]|, the scale a
 * comparison of out should be judged against, since the signed sum can cancel.
 */
void vatp_oracle_attention_output(const double *q, const double *K, const double *V, int64_t n,
                                  int64_t d, double c, double *out, double *abs_out,
                                  double *scratch)
{
    double m = -INFINITY;
    for (int64_t r = 0; r < n; ++r) {
        double dot = 0.0;
        for (int64_t x = 0; x < d; ++x) dot += q[x] * K[r * d + x];
        scratch[r] = c * dot;
        if (scratch[r] > m) m = scratch[r];
    }
    double denom = 0.0;
    for (int64_t r = 0; r < n; ++r) {
        scratch[r] = exp(scratch[r] - m);
        denom += scratch[r];
    }
    for (int64_t x = 0; x < d; ++x) {
        double s = 0.0, sa = 0.0;
        for (int64_t r = 0; r < n; ++r) {
            double a = scratch[r] / denom;
            s += a * V[r * d + x];
            sa += a * fabs(V[r * d + x]);
        }
        out[x] = s;
        if (abs_out) abs_out[x] = sa;
    }
}

/* l1 norm of each value row (the norm used in Eq. 4).  V: [n, d] -> nrm: [n]. */
void vatp_oracle_l1norm(const double *V, int64_t n, int64_t d, double *nrm)
{
    for (int64_t r = 0; r < n; ++r) {
        double s = 0.0;
        for (int64_t x = 0; x < d; ++x) s += fabs(V[r * d + x]);
        nrm[r] = s;
    }
}

/*
 * Attention score over a history window of w steps (Eq. 3), after a causal prompt pass
 * (t = L-1):
 *     S_i = sum_{j = max(L-1-w, i)}^{L-1} a_i^j ,
 * with a^j the same softmax rows as above.  Also returns those rows themselves, oldest first:
 * P[r][i] = a_i^{j0+r}, j0 = max(0, L-1-w), r < n_hist = L - j0 (zero for i > j0+r); a later
 * step needs them to drop the row that leaves the window.  Q, K: [L, d].  S: [L].
 * P: [n_hist, L].  scratch: [L].  Returns n_hist.
 */
int64_t vatp_oracle_prefill_window(const double *Q, const double *K, int64_t L, int64_t d, double c,
                                   int64_t w, double *S, double *P, double *scratch)
{
    const int64_t j0 = L - 1 - w > 0 ? L - 1 - w : 0;
    for (int64_t i = 0; i < L; ++i) S[i] = 0.0;
    for (int64_t j = j0; j < L; ++j) {
        const double *q = Q + j * d;
        double *row = P + (j - j0) * L;
        double m = -INFINITY;
        for (int64_t i = 0; i <= j; ++i) {
            const double *k = K + i * d;
            double dot = 0.0;
            for (int64_t x = 0; x < d; ++x) dot += q[x] * k[x];
            scratch[i] = c * dot;
            if (scratch[i] > m) m = scratch[i];
        }
        double denom = 0.0;
        for (int64_t i = 0; i <= j; ++i) {
            scratch[i] = exp(scratch[i] - m);
            denom += scratch[i];
        }
        for (int64_t i = 0; i < L; ++i) row[i] = i <= j ? scratch[i] / denom : 0.0;
        for (int64_t i = 0; i <= j; ++i) S[i] += row[i];
    }
    return L - j0;
}

/*
 * The norm ablation (Table 2): kind 0 = l1 (the paper's choice, same as above),
 * 1 = l2 = sqrt(sum v^2), 2 = l-infinity = max |v|.  V: [n, d] -> nrm: [n].
 */
void vatp_oracle_vnorm(const double *V, int64_t n, int64_t d, int kind, double *nrm)
{
    for (int64_t r = 0; r < n; ++r) {
        double s = 0.0;
        for (int64_t x = 0; x < d; ++x) {
            double a = fabs(V[r * d + x]);
            if (kind == 0) s += a;
            else if (kind == 1) s += a * a;
            else if (a > s) s = a;
        }
        nrm[r] = kind == 1 ? sqrt(s) : kind == 3 ? 1.0 : s;
    }
}

/*
 * Value-aware importance, Eq. 4:  I_r = S_r * ||v_r||_1.
 */
void vatp_oracle_importance(const double *S, const double *nrm, int64_t n, double *I)
{
    for (int64_t r = 0; r < n; ++r) I[r] = S[r] * nrm[r];
}

/*
 * Budgeted selection on a cache of n rows (Attention Sink Tokens paragraph for the
 * forced prefix F; Implementation Details appendix for the budget split into
 * importance-selected rows plus a local window of the most recent rows).
 *   n <= B : every row is kept.
 *   else   : rows [0,F) and [n-R,n) are kept unconditionally; of the candidates
 *            [F, n-R) the B-F-R with the largest I are kept, equal I resolved in
 *            favour of the lower row index.
 * kept (size >= min(n,B)) receives the surviving row indices in ascending order.
 * Returns the number of rows kept, or -1 if B < F + R.
 */
int64_t vatp_oracle_select(const double *I, int64_t n, int64_t B, int64_t F, int64_t R,
                           int32_t *kept)
{
    if (B < F + R) return -1;
    if (n <= B) {
        for (int64_t r = 0; r < n; ++r) kept[r] = (int32_t)r;
        return n;
    }
    int64_t n_heavy = B - F - R;
    int64_t lo = F, hi = n - R;            /* candidates are rows lo .. hi-1 */
    char *keep = (char *)calloc((size_t)n, 1);
    for (int64_t r = 0; r < lo; ++r) keep[r] = 1;
    for (int64_t r = hi; r < n; ++r) keep[r] = 1;
    /* pick the n_heavy best candidates one at a time: largest I, lowest index first */
    for (int64_t pick = 0; pick < n_heavy; ++pick) {
        int64_t best = -1;
        for (int64_t r = lo; r < hi; ++r) {
            if (keep[r]) continue;
            if (best < 0 || I[r] > I[best]) best = r;   /* strict '>' keeps the lower index */
        }
        keep[best] = 1;
    }
    int64_t out = 0;
    for (int64_t r = 0; r < n; ++r)
        if (keep[r]) kept[out++] = (int32_t)r;
    free(keep);
    return out;
}

/* Compaction: out row o = in row kept[o].  Rows are `width` doubles wide. */
void vatp_oracle_gather_rows(const double *in, const int32_t *kept, int64_t n_kept,
                             int64_t width, double *out)
{
    for (int64_t o = 0; o < n_kept; ++o)
        memcpy(out + o * width, in + (int64_t)kept[o] * width, (size_t)width * sizeof(double));
}

/* ---- drivers over independent (sequence, head) units; used for CPU timing ---- */

/* Q, K: [units, cap, d]; len[u] rows valid; S: [units, cap]. */
void vatp_oracle_prefill_scores_units(const double *Q, const double *K, int64_t units,
                                      int64_t cap, const int64_t *len, int64_t d, double c,
                                      double *S)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        double *scratch = (double *)malloc((size_t)(len[u] > 0 ? len[u] : 1) * sizeof(double));
        vatp_oracle_prefill_scores(Q + u * cap * d, K + u * cap * d, len[u], d, c,
                                   S + u * cap, scratch);
        free(scratch);
    }
}

/*
 * One decode-and-prune step for every unit, out of place:
 * (K,V,S,nrm) hold n[u] rows that already include the appended token (S of that row 0).
 * Scores are updated with q, importance formed, selection taken, survivors gathered
 * into the *_out arrays; n_out[u] receives the new row count.
 */
void vatp_oracle_decode_prune_units(const double *q, const double *K, const double *V,
                                    double *S, const double *nrm, int64_t units, int64_t cap,
                                    const int64_t *n, int64_t d, double c, const int64_t *B,
                                    int64_t F, int64_t R, double *K_out, double *V_out,
                                    double *S_out, double *nrm_out, int32_t *kept,
                                    int64_t *n_out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        int64_t nu = n[u];
        double *scratch = (double *)malloc((size_t)(nu > 0 ? nu : 1) * sizeof(double));
        double *I = (double *)malloc((size_t)(nu > 0 ? nu : 1) * sizeof(double));
        vatp_oracle_decode_scores(q + u * d, K + u * cap * d, nu, d, c, S + u * cap, NULL, scratch);
        vatp_oracle_importance(S + u * cap, nrm + u * cap, nu, I);
        int64_t nk = vatp_oracle_select(I, nu, B[u], F, R, kept + u * cap);
        n_out[u] = nk;
        if (nk >= 0) {
            vatp_oracle_gather_rows(K + u * cap * d, kept + u * cap, nk, d, K_out + u * cap * d);
            vatp_oracle_gather_rows(V + u * cap * d, kept + u * cap, nk, d, V_out + u * cap * d);
            vatp_oracle_gather_rows(S + u * cap, kept + u * cap, nk, 1, S_out + u * cap);
            vatp_oracle_gather_rows(nrm + u * cap, kept + u * cap, nk, 1, nrm_out + u * cap);
        }
        free(I);
        free(scratch);
    }
}

int vatp_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
