/*
 * Sanitizer driver for the CPU oracle (test infrastructure): built together with ssn_oracle.c under
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py, it calls every entry point of the oracle on a
 * small dense and a small CSR problem (empty rows, repeated sample rows, the reference class, K = 1), so that an
 * out-of-bounds access, a leak or undefined arithmetic in the oracle aborts the run.  It checks no values: the
 * pins of tests/test_oracle_*.py do that.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int64_t n, p;
    int32_t C;
    int32_t scale_sum;
    double lambda;
    const double *X;
    int64_t ldx;
    const int64_t *rowptr;
    const int32_t *colidx;
    const double *vals;
    const int32_t *labels;
} orc_problem;

double orc_objective(const orc_problem *, const double *);
void orc_row_parts(const orc_problem *, const double *, double *, double *, double *, double *);
void orc_gradient(const orc_problem *, const double *, double *, double *);
void orc_gradient_sampled(const orc_problem *, const double *, const int32_t *, int64_t, double *, double *);
void orc_sample_probs(const orc_problem *, const double *, const int32_t *, int64_t, double *);
void orc_hessvec(const orc_problem *, const double *, const int32_t *, int64_t, const double *, double *);
void orc_predict(const orc_problem *, const double *, int32_t *);
double orc_accuracy(const orc_problem *, const double *);
int orc_cg(const orc_problem *, const double *, const int32_t *, int64_t, const double *, double, int, double *, double *,
           int32_t *, double *);
int orc_linesearch(const orc_problem *, const double *, const double *, const double *, double, double, double, int,
                   double *, double *, int32_t *);
int orc_ssn(const orc_problem *, double *, int, const int32_t *, int64_t, double, double, int, double, double, int, double *);
int orc_ssn_sg(const orc_problem *, double *, int, const int32_t *, int64_t, const int32_t *, int64_t, double, double, int,
               double, double, int, double *);
void orc_normalize_columns(int64_t, int64_t, double *, int64_t, const int64_t *, const int32_t *, double *, double *);
int orc_threads(void);

static uint64_t state = 88172645463325252ULL;
static double rnd(void)                     /* xorshift, uniform in (-1, 1) */
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}

static void exercise(const orc_problem *pr, int iters)
{
    const int K = pr->C - 1;
    const int64_t d = pr->p * K, n = pr->n;
    double *W = malloc(sizeof(double) * d), *V = malloc(sizeof(double) * d), *G = malloc(sizeof(double) * d);
    double *HV = malloc(sizeof(double) * d), *P = malloc(sizeof(double) * d);
    for (int64_t t = 0; t < d; ++t) { W[t] = 0.3 * rnd(); V[t] = rnd(); }
    const int64_t nS = n / 3 + 1;
    int32_t *S = malloc(sizeof(int32_t) * nS * iters), *pred = malloc(sizeof(int32_t) * n);
    for (int64_t s = 0; s < nS * iters; ++s) S[s] = (int32_t)((s * 7) % n);
    S[1] = S[0];                                        /* a repeated row */
    double *parts = malloc(sizeof(double) * 4 * n), *probs = malloc(sizeof(double) * nS * K), f, fs, rel, alpha, fn;
    double *trace = malloc(sizeof(double) * 3 * 12), *log = malloc(sizeof(double) * 6 * iters);
    int32_t flags, ok;
    (void)orc_objective(pr, W);
    orc_row_parts(pr, W, parts, parts + n, parts + 2 * n, parts + 3 * n);
    orc_gradient(pr, W, G, &f);
    orc_gradient_sampled(pr, W, S, nS, HV, &fs);
    orc_sample_probs(pr, W, S, nS, probs);
    orc_hessvec(pr, W, S, nS, V, HV);
    orc_predict(pr, W, pred);
    (void)orc_accuracy(pr, W);
    (void)orc_cg(pr, W, S, nS, G, 1e-6, 12, P, &rel, &flags, trace);
    (void)orc_cg(pr, W, S, nS, G, 1e-6, 0, P, &rel, &flags, NULL);
    (void)orc_linesearch(pr, W, P, G, f, 1e-4, 0.5, 10, &alpha, &fn, &ok);
    for (int64_t t = 0; t < d; ++t) W[t] = 0.0;
    (void)orc_ssn(pr, W, iters, S, nS, 0.0, 1e-4, 5, 1e-4, 0.5, 10, log);
    for (int64_t t = 0; t < d; ++t) W[t] = 0.0;
    (void)orc_ssn_sg(pr, W, iters, S, nS, S, nS, 0.0, 1e-4, 5, 1e-4, 0.5, 10, log);
    free(log); free(trace); free(probs); free(parts); free(pred); free(S);
    free(P); free(HV); free(G); free(V); free(W);
}

int main(void)
{
    const int64_t n = 57, p = 11;
    for (int C = 2; C <= 5; C += 3) {
        /* dense */
        double *X = malloc(sizeof(double) * n * p), *norm = malloc(sizeof(double) * p);
        int32_t *lab = malloc(sizeof(int32_t) * n);
        for (int64_t t = 0; t < n * p; ++t) X[t] = rnd();
        for (int64_t i = 0; i < n; ++i) lab[i] = (int32_t)(i % C);
        orc_normalize_columns(n, p, X, p, NULL, NULL, NULL, norm);
        orc_problem pd = {n, p, C, 0, 1e-2, X, p, NULL, NULL, NULL, lab};
        exercise(&pd, 3);
        pd.scale_sum = 1;
        exercise(&pd, 2);
        /* CSR with empty rows */
        int64_t *rowptr = malloc(sizeof(int64_t) * (n + 1));
        int32_t *col = malloc(sizeof(int32_t) * n * 4);
        double *val = malloc(sizeof(double) * n * 4);
        int64_t nnz = 0;
        rowptr[0] = 0;
        for (int64_t i = 0; i < n; ++i) {
            const int k = (i % 5 == 0) ? 0 : (int)(1 + i % 4);
            for (int j = 0; j < k; ++j) { col[nnz] = (int32_t)((i + 3 * j) % p); val[nnz] = rnd(); ++nnz; }
            rowptr[i + 1] = nnz;
        }
        orc_normalize_columns(n, p, NULL, 0, rowptr, col, val, norm);
        orc_problem ps = {n, p, C, 0, 1e-2, NULL, 0, rowptr, col, val, lab};
        exercise(&ps, 3);
        free(val); free(col); free(rowptr); free(lab); free(norm); free(X);
    }
    printf("sanitize_check ok (%d thread%s)\n", orc_threads(), orc_threads() == 1 ? "" : "s");
    return 0;
}
