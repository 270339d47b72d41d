/*
 * Host sanitizer pass over the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Built together with scfa_oracle.c under -fsanitize=address,undefined and run by
 * tests/test_oracle_sanitizers.py: every entry point of the oracle is driven with small seeded inputs that
 * include the edge cases of the method (T = 1, rows without any allowed key, nothing kept, strict causality,
 * row subsets given in scrambled order).  The program checks two invariants on the way (probability rows
 * sum to 1 or 0; the pair count equals the number of non-zero probabilities) and exits 0; any out-of-bounds
 * access, use of uninitialised heap, signed overflow or misaligned access aborts it with a report.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void scfa_oracle_forward_rows(const double *Q, const double *K, const double *V, const int32_t *lab_q,
                              const int32_t *lab_k, int variant, int strict, int T, int d, double tau,
                              const int32_t *rows, int nrows, double *O_rows, double *LSE_rows, double *m_rows,
                              double *l_rows);
void scfa_oracle_probs(const double *Q, const double *K, const int32_t *lab_q, const int32_t *lab_k, int variant,
                       int strict, int T, int d, double tau, double *P);
void scfa_oracle_row_stats(const double *Q, const double *K, const double *V, const double *dO, const int32_t *lab_q,
                           const int32_t *lab_k, int variant, int strict, int T, int d, double tau, double *m_all,
                           double *l_all, double *D_all);
void scfa_oracle_dq_rows(const double *Q, const double *K, const double *V, const double *dO, const int32_t *lab_q,
                         const int32_t *lab_k, int variant, int strict, int T, int d, double tau, const int32_t *rows,
                         int nrows, double *dQ_rows);
void scfa_oracle_dkdv_rows(const double *Q, const double *K, const double *V, const double *dO, const int32_t *lab_q,
                           const int32_t *lab_k, int variant, int strict, int T, int d, double tau, const double *m_all,
                           const double *l_all, const double *D_all, const int32_t *rows, int nrows, double *dK_rows,
                           double *dV_rows);
long long scfa_oracle_count_pairs(const int32_t *lab_q, const int32_t *lab_k, int variant, int strict, int T);

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double uniform(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static double *alloc_random(size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = 4.0 * uniform() - 2.0;
    return p;
}

/* mode 0: hash with nb labels; 1: keep flags with the given rate; 2: nothing kept on the key side */
static int run_case(int variant, int strict, int T, int d, int nb, double keep, int mode)
{
    double *Q = alloc_random((size_t)T * d), *K = alloc_random((size_t)T * d), *V = alloc_random((size_t)T * d),
           *dO = alloc_random((size_t)T * d);
    int32_t *lq = (int32_t *)malloc(sizeof(int32_t) * T), *lk = (int32_t *)malloc(sizeof(int32_t) * T);
    for (int t = 0; t < T; ++t) {
        if (mode == 0) { lq[t] = (int32_t)(uniform() * nb); lk[t] = (int32_t)(uniform() * nb); }
        else { lq[t] = uniform() < keep; lk[t] = mode == 2 ? 0 : uniform() < keep; }
    }
    /* every other row, in descending order, plus row 0 twice */
    int nrows = 0;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (T + 2));
    for (int t = T - 1; t >= 0; t -= 2) rows[nrows++] = t;
    rows[nrows++] = 0; rows[nrows++] = 0;
    double *O = alloc_random((size_t)nrows * d), *LSE = alloc_random(nrows), *m = alloc_random(nrows), *l = alloc_random(nrows);
    const double tau = 1.0 / sqrt((double)d);
    scfa_oracle_forward_rows(Q, K, V, lq, lk, variant, strict, T, d, tau, rows, nrows, O, LSE, m, l);
    scfa_oracle_forward_rows(Q, K, V, lq, lk, variant, strict, T, d, tau, rows, nrows, O, LSE, NULL, NULL);
    double *P = alloc_random((size_t)T * T);
    scfa_oracle_probs(Q, K, lq, lk, variant, strict, T, d, tau, P);
    long long nonzero = 0;
    int bad = 0;
    for (int i = 0; i < T; ++i) {
        double sum = 0.0;
        for (int j = 0; j < T; ++j) { sum += P[(size_t)i * T + j]; nonzero += P[(size_t)i * T + j] != 0.0; }
        if (!(fabs(sum - 1.0) < 1e-12 || sum == 0.0)) bad = 1;
    }
    if (nonzero != scfa_oracle_count_pairs(lq, lk, variant, strict, T)) bad = 1;
    double *m_all = alloc_random(T), *l_all = alloc_random(T), *D_all = alloc_random(T);
    scfa_oracle_row_stats(Q, K, V, dO, lq, lk, variant, strict, T, d, tau, m_all, l_all, D_all);
    double *dQ = alloc_random((size_t)nrows * d), *dK = alloc_random((size_t)nrows * d), *dV = alloc_random((size_t)nrows * d);
    scfa_oracle_dq_rows(Q, K, V, dO, lq, lk, variant, strict, T, d, tau, rows, nrows, dQ);
    scfa_oracle_dkdv_rows(Q, K, V, dO, lq, lk, variant, strict, T, d, tau, m_all, l_all, D_all, rows, nrows, dK, dV);
    for (size_t i = 0; i < (size_t)nrows * d; ++i)
        if (!isfinite(O[i]) || !isfinite(dQ[i]) || !isfinite(dK[i]) || !isfinite(dV[i])) bad = 1;
    free(Q); free(K); free(V); free(dO); free(lq); free(lk); free(rows); free(O); free(LSE); free(m); free(l);
    free(P); free(m_all); free(l_all); free(D_all); free(dQ); free(dK); free(dV);
    return bad;
}

int main(void)
{
    int bad = 0, cases = 0;
    const int Ts[] = {1, 2, 7, 64, 129};
    for (unsigned ti = 0; ti < sizeof(Ts) / sizeof(Ts[0]); ++ti)
        for (int strict = 0; strict < 2; ++strict) {
            bad |= run_case(0, strict, Ts[ti], 8, 1, 0.0, 0); ++cases;      /* one bucket: dense causal */
            bad |= run_case(0, strict, Ts[ti], 5, 4, 0.0, 0); ++cases;      /* four buckets, odd head dimension */
            bad |= run_case(0, strict, Ts[ti], 4, 300, 0.0, 0); ++cases;    /* more buckets than tokens */
            bad |= run_case(1, strict, Ts[ti], 8, 1, 0.5, 1); ++cases;      /* half kept */
            bad |= run_case(1, strict, Ts[ti], 8, 1, 1.0, 1); ++cases;      /* all kept */
            bad |= run_case(1, strict, Ts[ti], 8, 1, 0.5, 2); ++cases;      /* no key kept */
        }
    printf("oracle sanitizer pass: %d cases, invariants %s\n", cases, bad ? "VIOLATED" : "hold");
    return bad;
}
