/*
 * CPU oracle for Sparse Causal Flash Attention -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It is never linked into, imported by, or called from the product
 * path; it shares no code, header, table or helper with the HIP sources.
 *
 * What it computes (paper Sec. 3: the method is exact, not an approximation): the
 * method's result is exact softmax attention restricted to a mask, so the
 * oracle is that definition written out on the ORIGINAL, unpermuted tensors,
 * in double precision, with a two-pass softmax per row.  It never sorts,
 * compacts, tiles, or keeps running statistics.
 *
 *   allowed(i,j) = (j <= i)                       causal, inclusive (Sec. 3.1: the tile rule
 *                                                 skips only max(q_idx) < min(k_idx); App. B.1
 *                                                 mask "q_idx >= k_idx"; Fig. 1 row counts)
 *                  AND  hash   : label_q[i] == label_k[j]      (Sec. 3.2, App. B.1 mask)
 *                       qkdrop : keep_q[i] != 0 AND keep_k[j] != 0   (Sec. 3.1)
 *   s_ij = tau * <Q_i, K_j>                       (Alg. 1 / Alg. 2 "inner product")
 *   m_i  = max_j s_ij,  l_i = sum_j exp(s_ij - m_i)       over allowed j
 *   P_ij = exp(s_ij - m_i) / l_i,   O_i = sum_j P_ij V_j,   LSE_i = m_i + ln l_i
 *   a row with no allowed key: O_i = 0, P_i. = 0 (Sec. 3.1 "Edge cases":
 *   stranded queries default to zero vectors); LSE_i = -inf is this build's
 *   reading (ln 0) -- the paper does not state it: parity unpinned for that
 *   one value.
 *
 * Backward (the paper only says the backward is adapted "in a similar
 * fashion"; these are the derivatives of the definition above, given dO):
 *   dP_ij = <dO_i, V_j>          D_i = sum_j P_ij dP_ij
 *   dS_ij = P_ij (dP_ij - D_i)   (0 where not allowed)
 *   dQ_i  = tau sum_j dS_ij K_j
 *   dK_j  = tau sum_i dS_ij Q_i
 *   dV_j  = sum_i P_ij dO_i
 * D is computed from sum_j P dP (not from <dO_i,O_i>) so that identity is a
 * test, not an assumption.
 *
 * `strict` != 0 replaces (j <= i) by (j < i): the variant App. B.1 mentions
 * ("we often replace >= by >").
 *
 * All functions work on ONE (batch, head) segment; the Python wrapper loops
 * over segments.  Every output element is produced by its own plain sum in
 * index order, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SCFA_ORACLE_HASH 0
#define SCFA_ORACLE_QKDROP 1

static int pair_allowed(int variant, int strict, int i, int j,
                        const int32_t *lab_q, const int32_t *lab_k)
{
    if (strict ? (j >= i) : (j > i)) return 0;
    if (variant == SCFA_ORACLE_HASH) return lab_q[i] == lab_k[j];
    return lab_q[i] != 0 && lab_k[j] != 0;
}

static double dot(const double *a, const double *b, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += a[c] * b[c];
    return acc;
}

/* scores of row i into s[0..T) (only allowed entries are written), returns
 * the number of allowed keys and the row maximum through *m_out. */
static int row_scores(const double *Q, const double *K, const int32_t *lab_q,
                      const int32_t *lab_k, int variant, int strict, int T, int d,
                      double tau, int i, double *s, double *m_out)
{
    int n = 0;
    double m = -INFINITY;
    (void)T;
    for (int j = 0; j <= i; ++j) {
        if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
        s[j] = tau * dot(Q + (size_t)i * d, K + (size_t)j * d, d);
        if (s[j] > m) m = s[j];
        ++n;
    }
    *m_out = m;
    return n;
}

/* Forward for the listed rows.  O_rows [nrows,d], LSE_rows [nrows];
 * m_rows / l_rows (nullable) receive the row maximum and the row sum. */
void scfa_oracle_forward_rows(const double *Q, const double *K, const double *V,
                              const int32_t *lab_q, const int32_t *lab_k,
                              int variant, int strict, int T, int d, double tau,
                              const int32_t *rows, int nrows,
                              double *O_rows, double *LSE_rows,
                              double *m_rows, double *l_rows)
{
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)T);
#pragma omp for schedule(dynamic, 8)
        for (int r = 0; r < nrows; ++r) {
            const int i = rows[r];
            double *o = O_rows + (size_t)r * d;
            double m;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            const int n = row_scores(Q, K, lab_q, lab_k, variant, strict, T, d, tau, i, s, &m);
            if (n == 0) {
                LSE_rows[r] = -INFINITY;
                if (m_rows) m_rows[r] = -INFINITY;
                if (l_rows) l_rows[r] = 0.0;
                continue;
            }
            double l = 0.0;
            for (int j = 0; j <= i; ++j)
                if (pair_allowed(variant, strict, i, j, lab_q, lab_k)) l += exp(s[j] - m);
            for (int j = 0; j <= i; ++j) {
                if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
                const double p = exp(s[j] - m) / l;
                const double *v = V + (size_t)j * d;
                for (int c = 0; c < d; ++c) o[c] += p * v[c];
            }
            LSE_rows[r] = m + log(l);
            if (m_rows) m_rows[r] = m;
            if (l_rows) l_rows[r] = l;
        }
        free(s);
    }
}

/* Dense probability matrix P [T,T] (row-major, zeros where masked); for small T. */
void scfa_oracle_probs(const double *Q, const double *K,
                       const int32_t *lab_q, const int32_t *lab_k,
                       int variant, int strict, int T, int d, double tau, double *P)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)T);
    for (int i = 0; i < T; ++i) {
        double m;
        double *p = P + (size_t)i * T;
        for (int j = 0; j < T; ++j) p[j] = 0.0;
        const int n = row_scores(Q, K, lab_q, lab_k, variant, strict, T, d, tau, i, s, &m);
        if (n == 0) continue;
        double l = 0.0;
        for (int j = 0; j <= i; ++j)
            if (pair_allowed(variant, strict, i, j, lab_q, lab_k)) l += exp(s[j] - m);
        for (int j = 0; j <= i; ++j)
            if (pair_allowed(variant, strict, i, j, lab_q, lab_k)) p[j] = exp(s[j] - m) / l;
    }
    free(s);
}

/* Per-row statistics needed by the key-side gradients: m_i, l_i and
 * D_i = sum_j P_ij <dO_i, V_j>, for every row of the segment. */
void scfa_oracle_row_stats(const double *Q, const double *K, const double *V, const double *dO,
                           const int32_t *lab_q, const int32_t *lab_k,
                           int variant, int strict, int T, int d, double tau,
                           double *m_all, double *l_all, double *D_all)
{
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)T);
#pragma omp for schedule(dynamic, 8)
        for (int i = 0; i < T; ++i) {
            double m;
            const int n = row_scores(Q, K, lab_q, lab_k, variant, strict, T, d, tau, i, s, &m);
            if (n == 0) { m_all[i] = -INFINITY; l_all[i] = 0.0; D_all[i] = 0.0; continue; }
            double l = 0.0;
            for (int j = 0; j <= i; ++j)
                if (pair_allowed(variant, strict, i, j, lab_q, lab_k)) l += exp(s[j] - m);
            double D = 0.0;
            for (int j = 0; j <= i; ++j) {
                if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
                const double p = exp(s[j] - m) / l;
                D += p * dot(dO + (size_t)i * d, V + (size_t)j * d, d);
            }
            m_all[i] = m; l_all[i] = l; D_all[i] = D;
        }
        free(s);
    }
}

/* dQ for the listed query rows.  dQ_rows [nrows,d]. */
void scfa_oracle_dq_rows(const double *Q, const double *K, const double *V, const double *dO,
                         const int32_t *lab_q, const int32_t *lab_k,
                         int variant, int strict, int T, int d, double tau,
                         const int32_t *rows, int nrows, double *dQ_rows)
{
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)T);
        double *dp = (double *)malloc(sizeof(double) * (size_t)T);
#pragma omp for schedule(dynamic, 8)
        for (int r = 0; r < nrows; ++r) {
            const int i = rows[r];
            double *dq = dQ_rows + (size_t)r * d;
            double m;
            for (int c = 0; c < d; ++c) dq[c] = 0.0;
            const int n = row_scores(Q, K, lab_q, lab_k, variant, strict, T, d, tau, i, s, &m);
            if (n == 0) continue;
            double l = 0.0;
            for (int j = 0; j <= i; ++j)
                if (pair_allowed(variant, strict, i, j, lab_q, lab_k)) l += exp(s[j] - m);
            double D = 0.0;
            for (int j = 0; j <= i; ++j) {
                if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
                dp[j] = dot(dO + (size_t)i * d, V + (size_t)j * d, d);
                D += exp(s[j] - m) / l * dp[j];
            }
            for (int j = 0; j <= i; ++j) {
                if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
                const double p = exp(s[j] - m) / l;
                const double ds = p * (dp[j] - D);
                const double *k = K + (size_t)j * d;
                for (int c = 0; c < d; ++c) dq[c] += tau * ds * k[c];
            }
        }
        free(s);
        free(dp);
    }
}

/* dK and dV for the listed key rows, given the row statistics of the whole
 * segment (scfa_oracle_row_stats).  dK_rows, dV_rows [nrows,d]. */
void scfa_oracle_dkdv_rows(const double *Q, const double *K, const double *V, const double *dO,
                           const int32_t *lab_q, const int32_t *lab_k,
                           int variant, int strict, int T, int d, double tau,
                           const double *m_all, const double *l_all, const double *D_all,
                           const int32_t *rows, int nrows, double *dK_rows, double *dV_rows)
{
#pragma omp parallel for schedule(dynamic, 8)
    for (int r = 0; r < nrows; ++r) {
        const int j = rows[r];
        double *dk = dK_rows + (size_t)r * d;
        double *dv = dV_rows + (size_t)r * d;
        for (int c = 0; c < d; ++c) { dk[c] = 0.0; dv[c] = 0.0; }
        for (int i = j; i < T; ++i) {
            if (!pair_allowed(variant, strict, i, j, lab_q, lab_k)) continue;
            const double sij = tau * dot(Q + (size_t)i * d, K + (size_t)j * d, d);
            const double p = exp(sij - m_all[i]) / l_all[i];
            const double dpij = dot(dO + (size_t)i * d, V + (size_t)j * d, d);
            const double ds = p * (dpij - D_all[i]);
            const double *q = Q + (size_t)i * d;
            const double *g = dO + (size_t)i * d;
            for (int c = 0; c < d; ++c) { dk[c] += tau * ds * q[c]; dv[c] += p * g[c]; }
        }
    }
}

/* Number of allowed (query, key) pairs of a segment -- the "useful pair"
 * count used when a throughput is quoted per allowed pair. */
long long scfa_oracle_count_pairs(const int32_t *lab_q, const int32_t *lab_k,
                                  int variant, int strict, int T)
{
    long long total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int i = 0; i < T; ++i)
        for (int j = 0; j <= i; ++j)
            total += pair_allowed(variant, strict, i, j, lab_q, lab_k);
    return total;
}
