/*
 * CPU oracle for sub-sampled Newton on L2-regularised multinomial logistic
 * regression ("GPU Accelerated Sub-Sampled Newton's Method", arXiv 1802.09113).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow fp64
 * implementation whose only job is to be obviously correct so that the GPU
 * library can be checked against it.  Built as it is, it runs on one thread.
 * Built with -fopenmp (a second library, for the all-cores timing of the
 * benchmark and the long full-size test cases) the loops over rows of
 * objective, gradient and Hessian-vector product are cut into one contiguous
 * chunk of rows per thread, every thread sums its chunk exactly as the
 * single-thread loop would, and the per-thread sums are added in thread order;
 * tests/test_oracle_threads.py pins that build to the single-thread one.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may load it.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * Every function follows a passage of the paper:
 *   margins / stable log-sum-exp ......... Sec. 3.3.1 "Numerical Stability", eq. (8), (9)
 *   objective ............................ eq. (5); Alg. 5 with eqs. (14)-(17)
 *   gradient ............................. eq. (6); Alg. 6
 *   Hessian-vector product ............... eqs. (10)-(13); Alg. 7, Alg. 8
 *   sub-sampled Hessian .................. eq. (2b)
 *   sub-sampled gradient ................. eq. (2a)
 *   conjugate gradient ................... Alg. 2
 *   back-tracking line search ............ Alg. 3, eq. (3c)
 *   sub-sampled Newton iteration ......... Alg. 1, eq. (3a)
 *   classification rule .................. end of Sec. 3.3 (argmax over the C class probabilities)
 *   unit-column-norm preprocessing ....... Sec. 4 (columns divided by their 2-norms)
 *
 * Conventions (interface choices, stated here because the paper leaves them open):
 *   - n rows, p features, C classes, K = C-1.  Labels are 0-based in [0,C);
 *     label c < K belongs to weight column c, label C-1 is the reference class
 *     whose margin is identically zero (the paper's class C, x_c = w_c - w_C).
 *   - W, V, G, HV are p-by-K, row-major with leading dimension exactly K
 *     (entry (j,c) at [j*K + c]).  This is the paper's vec(.) up to a fixed
 *     permutation, so every norm and inner product is unchanged.
 *   - scale_sum == 0 ("mean"): data term of f, grad f is multiplied by 1/n and
 *     the sampled Hessian data term by 1/|S|.  scale_sum == 1 ("sum", the
 *     paper's eq. (1), (2b)): factors 1 and n/|S|.  The regulariser
 *     (lambda/2)||W||^2 is never scaled.
 *   - The data matrix is either dense row-major (X != NULL, leading dimension
 *     ldx) or CSR (rowptr/colidx/vals); one row accessor serves both.
 *   - Sums over rows are accumulated in long double so that the oracle is the
 *     more accurate side of a 1e-10 comparison.
 *
 * parity pins: every function below is pinned by tests/test_oracle_*.py
 * (finite differences, brute-force Hessian from eq. (7a)/(7b), W=0 closed
 * forms, the C=2 binary-logistic closed form of Appendix A.1, textbook CG on a
 * tiny SPD system, Armijo bracketing).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads for a loop over `rows` rows with a d-element long-double accumulator per thread (0 if none):
 * all the OpenMP build is given, but never more than there are rows, and never more accumulators than
 * fit 2 GiB.  1 without OpenMP. */
static int loop_threads(int64_t rows, int64_t d)
{
#ifdef _OPENMP
    int64_t nt = omp_get_max_threads();
    if (nt > rows) nt = rows;
    if (d > 0) {
        const int64_t fit = ((int64_t)1 << 31) / (d * (int64_t)sizeof(long double));
        if (nt > fit) nt = fit;
    }
    return nt < 1 ? 1 : (int)nt;
#else
    (void)rows; (void)d;
    return 1;
#endif
}

static int this_thread(void)
{
#ifdef _OPENMP
    return omp_get_thread_num();
#else
    return 0;
#endif
}

/* rows [lo, hi) of thread t of nt: contiguous chunks in row order */
static void thread_rows(int64_t rows, int nt, int t, int64_t *lo, int64_t *hi)
{
    const int64_t per = (rows + nt - 1) / nt;
    *lo = per * t < rows ? per * t : rows;
    *hi = *lo + per < rows ? *lo + per : rows;
}

/* acc[0..d) += acc[t*d .. (t+1)*d) for t = 1..nt-1, in that order */
static void fold_threads(long double *acc, int64_t d, int nt)
{
    for (int t = 1; t < nt; ++t)
        for (int64_t e = 0; e < d; ++e)
            acc[e] += acc[(int64_t)t * d + e];
}

typedef struct {
    int64_t n, p;
    int32_t C;
    int32_t scale_sum;          /* 0: mean scaling, 1: the paper's sum scaling */
    double lambda;
    const double *X;            /* dense row-major n x p, or NULL for CSR */
    int64_t ldx;
    const int64_t *rowptr;      /* CSR: n+1 entries */
    const int32_t *colidx;      /* CSR: nnz entries */
    const double *vals;         /* CSR: nnz entries */
    const int32_t *labels;      /* n entries in [0,C) */
} orc_problem;

/* z_c = <a_i, m_c> for c = 0..K-1, where M is p x K row-major (ld K). */
static void row_margins(const orc_problem *pr, int64_t i, const double *M, double *z)
{
    const int K = pr->C - 1;
    for (int c = 0; c < K; ++c) {
        long double acc = 0.0L;
        if (pr->X) {
            const double *a = pr->X + i * pr->ldx;
            for (int64_t j = 0; j < pr->p; ++j)
                acc += (long double)a[j] * (long double)M[j * K + c];
        } else {
            for (int64_t t = pr->rowptr[i]; t < pr->rowptr[i + 1]; ++t)
                acc += (long double)pr->vals[t] * (long double)M[(int64_t)pr->colidx[t] * K + c];
        }
        z[c] = (double)acc;
    }
}

/* acc[j*K + c] += a_ij * u_c  (rank-one update with row i of the data matrix). */
static void row_outer_add(const orc_problem *pr, int64_t i, const double *u, long double *acc)
{
    const int K = pr->C - 1;
    if (pr->X) {
        const double *a = pr->X + i * pr->ldx;
        for (int64_t j = 0; j < pr->p; ++j)
            for (int c = 0; c < K; ++c)
                acc[j * K + c] += (long double)a[j] * (long double)u[c];
    } else {
        for (int64_t t = pr->rowptr[i]; t < pr->rowptr[i + 1]; ++t)
            for (int c = 0; c < K; ++c)
                acc[(int64_t)pr->colidx[t] * K + c] += (long double)pr->vals[t] * (long double)u[c];
    }
}

/* eq. (8): M = max{0, z_1..z_K};  eq. (9): alpha = e^{-M} + sum_c e^{z_c - M}.
 * Returns M, writes alpha and (optionally) the probabilities p_c = e^{z_c-M}/alpha. */
static double stable_softmax(int K, const double *z, double *alpha_out, double *prob)
{
    double M = 0.0;
    for (int c = 0; c < K; ++c)
        if (z[c] > M) M = z[c];
    double alpha = exp(-M);
    for (int c = 0; c < K; ++c)
        alpha += exp(z[c] - M);
    if (prob)
        for (int c = 0; c < K; ++c)
            prob[c] = exp(z[c] - M) / alpha;
    *alpha_out = alpha;
    return M;
}

static double data_scale_full(const orc_problem *pr)
{
    return pr->scale_sum ? 1.0 : 1.0 / (double)pr->n;
}

static double data_scale_sample(const orc_problem *pr, int64_t nS)
{
    return pr->scale_sum ? (double)pr->n / (double)nS : 1.0 / (double)nS;
}

static long double half_lambda_sqnorm(const orc_problem *pr, const double *W)
{
    const int64_t d = pr->p * (int64_t)(pr->C - 1);
    long double s = 0.0L;
    for (int64_t t = 0; t < d; ++t)
        s += (long double)W[t] * (long double)W[t];
    return 0.5L * (long double)pr->lambda * s;
}

/* Per-row parts of Alg. 5: maxPart (eq. 14), sumExpPart (eq. 15), linearPart
 * (eq. 16), logPart (eq. 17), written to four n-vectors (any may be NULL). */
void orc_row_parts(const orc_problem *pr, const double *W,
                   double *maxPart, double *sumExpPart, double *linPart, double *logPart)
{
    const int K = pr->C - 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)K);
    for (int64_t i = 0; i < pr->n; ++i) {
        row_margins(pr, i, W, z);
        double M = 0.0;
        for (int c = 0; c < K; ++c)
            if (z[c] > M) M = z[c];
        double se = 0.0;
        for (int c = 0; c < K; ++c)
            se += exp(z[c] - M);
        const int b = pr->labels[i];
        if (maxPart) maxPart[i] = M;
        if (sumExpPart) sumExpPart[i] = se;
        if (linPart) linPart[i] = (b < K) ? z[b] : 0.0;
        if (logPart) logPart[i] = log(exp(-M) + se);
    }
    free(z);
}

/* f(W) = scale * sum_i [ M_i + log(alpha_i) - sum_c 1(b_i=c) z_ic ] + (lambda/2)||W||^2 */
double orc_objective(const orc_problem *pr, const double *W)
{
    const int K = pr->C - 1;
    const int nt = loop_threads(pr->n, 0);
    long double *tot = (long double *)calloc((size_t)nt, sizeof(long double));
#pragma omp parallel num_threads(nt)
    {
        const int t = this_thread();
        int64_t lo, hi;
        thread_rows(pr->n, nt, t, &lo, &hi);
        double *z = (double *)malloc(sizeof(double) * (size_t)K);
        long double total = 0.0L;
        for (int64_t i = lo; i < hi; ++i) {
            row_margins(pr, i, W, z);
            double alpha;
            const double M = stable_softmax(K, z, &alpha, NULL);
            const int b = pr->labels[i];
            const double lin = (b < K) ? z[b] : 0.0;
            total += (long double)M + (long double)log(alpha) - (long double)lin;
        }
        tot[t] = total;
        free(z);
    }
    fold_threads(tot, 1, nt);
    const long double total = tot[0];
    free(tot);
    return (double)((long double)data_scale_full(pr) * total + half_lambda_sqnorm(pr, W));
}

/* G = scale * sum_i a_i (p_i - y_i)^T + lambda W ; optionally also f(W). */
void orc_gradient(const orc_problem *pr, const double *W, double *G, double *f_out)
{
    const int K = pr->C - 1;
    const int64_t d = pr->p * (int64_t)K;
    const int nt = loop_threads(pr->n, d);
    long double *acc = (long double *)calloc((size_t)d * (size_t)nt, sizeof(long double));
    long double *tot = (long double *)calloc((size_t)nt, sizeof(long double));
#pragma omp parallel num_threads(nt)
    {
        const int t = this_thread();
        int64_t lo, hi;
        thread_rows(pr->n, nt, t, &lo, &hi);
        double *z = (double *)malloc(sizeof(double) * (size_t)K);
        double *prob = (double *)malloc(sizeof(double) * (size_t)K);
        long double total = 0.0L;
        for (int64_t i = lo; i < hi; ++i) {
            row_margins(pr, i, W, z);
            double alpha;
            const double M = stable_softmax(K, z, &alpha, prob);
            const int b = pr->labels[i];
            total += (long double)M + (long double)log(alpha) - (long double)((b < K) ? z[b] : 0.0);
            if (b < K) prob[b] -= 1.0;          /* BInd_ic = p_ic - 1(b_i = c) */
            row_outer_add(pr, i, prob, acc + (int64_t)t * d);
        }
        tot[t] = total;
        free(prob); free(z);
    }
    fold_threads(acc, d, nt);
    fold_threads(tot, 1, nt);
    const long double s = (long double)data_scale_full(pr);
    for (int64_t t = 0; t < d; ++t)
        G[t] = (double)(s * acc[t] + (long double)pr->lambda * (long double)W[t]);
    if (f_out)
        *f_out = (double)(s * tot[0] + half_lambda_sqnorm(pr, W));
    free(tot); free(acc);
}

/* Sub-sampled gradient, eq. (2a): G = scale_S * sum_{i in S} a_i (p_i - y_i)^T + lambda W with the
 * sample scaling of the Hessian (n/|S| in the paper's sum form, 1/|S| in the mean form).  S is a
 * multiset.  f_out (optional) receives the objective of the same sample,
 * scale_S * sum_{i in S} f_i(W) + (lambda/2)||W||^2, whose gradient G is. */
void orc_gradient_sampled(const orc_problem *pr, const double *W, const int32_t *S, int64_t nS,
                          double *G, double *f_out)
{
    const int K = pr->C - 1;
    const int64_t d = pr->p * (int64_t)K;
    const int nt = loop_threads(nS, d);
    long double *acc = (long double *)calloc((size_t)d * (size_t)nt, sizeof(long double));
    long double *tot = (long double *)calloc((size_t)nt, sizeof(long double));
#pragma omp parallel num_threads(nt)
    {
        const int t = this_thread();
        int64_t lo, hi;
        thread_rows(nS, nt, t, &lo, &hi);
        double *z = (double *)malloc(sizeof(double) * (size_t)K);
        double *prob = (double *)malloc(sizeof(double) * (size_t)K);
        long double total = 0.0L;
        for (int64_t s = lo; s < hi; ++s) {
            const int64_t i = S[s];
            row_margins(pr, i, W, z);
            double alpha;
            const double M = stable_softmax(K, z, &alpha, prob);
            const int b = pr->labels[i];
            total += (long double)M + (long double)log(alpha) - (long double)((b < K) ? z[b] : 0.0);
            if (b < K) prob[b] -= 1.0;
            row_outer_add(pr, i, prob, acc + (int64_t)t * d);
        }
        tot[t] = total;
        free(prob); free(z);
    }
    fold_threads(acc, d, nt);
    fold_threads(tot, 1, nt);
    const long double sc = (long double)data_scale_sample(pr, nS);
    for (int64_t t = 0; t < d; ++t)
        G[t] = (double)(sc * acc[t] + (long double)pr->lambda * (long double)W[t]);
    if (f_out)
        *f_out = (double)(sc * tot[0] + half_lambda_sqnorm(pr, W));
    free(tot); free(acc);
}

/* Probabilities of the sampled rows: P is nS x K row-major (the matrix W of eq. (11)). */
void orc_sample_probs(const orc_problem *pr, const double *W, const int32_t *S, int64_t nS, double *P)
{
    const int K = pr->C - 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)K);
    for (int64_t s = 0; s < nS; ++s) {
        row_margins(pr, S[s], W, z);
        double alpha;
        (void)stable_softmax(K, z, &alpha, P + s * K);
    }
    free(z);
}

/* HV = scale_S * sum_{i in S} a_i u_i^T + lambda V, with (eq. 12 / Alg. 8)
 *   vhat_i = V^T a_i,  t_i = sum_c p_ic vhat_ic,  u_ic = p_ic vhat_ic - p_ic t_i.
 * S is a multiset: a repeated index is summed as often as it occurs. */
void orc_hessvec(const orc_problem *pr, const double *W, const int32_t *S, int64_t nS,
                 const double *V, double *HV)
{
    const int K = pr->C - 1;
    const int64_t d = pr->p * (int64_t)K;
    const int nt = loop_threads(nS, d);
    long double *acc = (long double *)calloc((size_t)d * (size_t)nt, sizeof(long double));
#pragma omp parallel num_threads(nt)
    {
        const int th = this_thread();
        int64_t lo, hi;
        thread_rows(nS, nt, th, &lo, &hi);
        double *z = (double *)malloc(sizeof(double) * (size_t)K);
        double *prob = (double *)malloc(sizeof(double) * (size_t)K);
        double *vhat = (double *)malloc(sizeof(double) * (size_t)K);
        double *u = (double *)malloc(sizeof(double) * (size_t)K);
        for (int64_t s = lo; s < hi; ++s) {
            const int64_t i = S[s];
            row_margins(pr, i, W, z);
            double alpha;
            (void)stable_softmax(K, z, &alpha, prob);
            row_margins(pr, i, V, vhat);
            double t = 0.0;
            for (int c = 0; c < K; ++c)
                t += vhat[c] * prob[c];
            for (int c = 0; c < K; ++c)
                u[c] = vhat[c] * prob[c] - prob[c] * t;
            row_outer_add(pr, i, u, acc + (int64_t)th * d);
        }
        free(u); free(vhat); free(prob); free(z);
    }
    fold_threads(acc, d, nt);
    const long double sc = (long double)data_scale_sample(pr, nS);
    for (int64_t t = 0; t < d; ++t)
        HV[t] = (double)(sc * acc[t] + (long double)pr->lambda * (long double)V[t]);
    free(acc);
}

/* argmax over [z_0 .. z_{K-1}, 0]; ties go to the lowest class index. */
void orc_predict(const orc_problem *pr, const double *W, int32_t *pred)
{
    const int K = pr->C - 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)K);
    for (int64_t i = 0; i < pr->n; ++i) {
        row_margins(pr, i, W, z);
        int best = 0;
        double bv = (K > 0) ? z[0] : 0.0;
        for (int c = 1; c < K; ++c)
            if (z[c] > bv) { bv = z[c]; best = c; }
        if (0.0 > bv) best = K;
        pred[i] = best;
    }
    free(z);
}

double orc_accuracy(const orc_problem *pr, const double *W)
{
    int32_t *pred = (int32_t *)malloc(sizeof(int32_t) * (size_t)pr->n);
    orc_predict(pr, W, pred);
    int64_t hit = 0;
    for (int64_t i = 0; i < pr->n; ++i)
        hit += (pred[i] == pr->labels[i]);
    free(pred);
    return (double)hit / (double)pr->n;
}

static long double ldot(int64_t d, const double *a, const double *b)
{
    long double s = 0.0L;
    for (int64_t t = 0; t < d; ++t)
        s += (long double)a[t] * (long double)b[t];
    return s;
}

/*
 * Alg. 2 (conjugate gradient with best-iterate memory) on H_S(W) p = -g.
 * At most T Hessian-vector products are made.  Returns the number of products.
 * trace (optional, 3*T doubles): per product k the step alpha_k, ||r_{k+1}|| and
 * s_k^T H s_k.  flags bit0: stopped by the theta test; bit1: s^T H s <= 0 met.
 */
/* Threads the row loops use: what the OpenMP build was given (OMP_NUM_THREADS), 1 in the plain build. */
int orc_threads(void)
{
    return loop_threads((int64_t)1 << 40, 0);
}

int orc_cg(const orc_problem *pr, const double *W, const int32_t *S, int64_t nS,
           const double *g, double theta, int T, double *p_best,
           double *rel_res_best, int32_t *flags, double *trace)
{
    const int64_t d = pr->p * (int64_t)(pr->C - 1);
    double *p = (double *)calloc((size_t)d, sizeof(double));
    double *r = (double *)malloc(sizeof(double) * (size_t)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)d);
    double *Hs = (double *)malloc(sizeof(double) * (size_t)d);
    double *r_best = (double *)malloc(sizeof(double) * (size_t)d);
    int fl = 0, nprod = 0;

    for (int64_t t = 0; t < d; ++t) {
        r[t] = -g[t];            /* r_0 = -g */
        s[t] = r[t];             /* s_0 = r_0 */
        p_best[t] = s[t];        /* p_best = s_0 */
        r_best[t] = r[t];        /* r_best = r_0 */
    }
    const double gnorm = sqrt((double)ldot(d, g, g));
    double rr = (double)ldot(d, r, r);
    double rbest_norm = sqrt(rr);

    if (gnorm == 0.0) {
        memset(p_best, 0, sizeof(double) * (size_t)d);
        T = 0;
    }
    for (int k = 0; k < T; ++k) {
        orc_hessvec(pr, W, S, nS, s, Hs);
        ++nprod;
        const double sHs = (double)ldot(d, s, Hs);
        if (!(sHs > 0.0)) { fl |= 2; if (trace) { trace[3*k] = 0; trace[3*k+1] = sqrt(rr); trace[3*k+2] = sHs; } break; }
        const double a = rr / sHs;
        for (int64_t t = 0; t < d; ++t) p[t] += a * s[t];
        for (int64_t t = 0; t < d; ++t) r[t] -= a * Hs[t];
        const double rr_new = (double)ldot(d, r, r);
        const double rnorm = sqrt(rr_new);
        if (trace) { trace[3*k] = a; trace[3*k+1] = rnorm; trace[3*k+2] = sHs; }
        if (rnorm <= rbest_norm) {
            rbest_norm = rnorm;
            memcpy(r_best, r, sizeof(double) * (size_t)d);
            memcpy(p_best, p, sizeof(double) * (size_t)d);
        }
        if (rnorm <= theta * gnorm) { fl |= 1; break; }
        const double b = rr_new / rr;
        for (int64_t t = 0; t < d; ++t) s[t] = r[t] + b * s[t];
        rr = rr_new;
    }
    if (rel_res_best) *rel_res_best = (gnorm > 0.0) ? rbest_norm / gnorm : 0.0;
    if (flags) *flags = fl;
    free(r_best); free(Hs); free(s); free(r); free(p);
    return nprod;
}

/*
 * Alg. 3: alpha = 1; while F(W + alpha P) > F(W) + alpha beta <P,g>:
 *            if i > i_max break; i += 1; alpha *= rho.
 * Returns the number of objective evaluations; *ok = 1 iff the loop ended with
 * the Armijo inequality satisfied.
 */
int orc_linesearch(const orc_problem *pr, const double *W, const double *P, const double *g,
                   double fW, double beta, double rho, int imax,
                   double *alpha_out, double *f_new, int32_t *ok)
{
    const int64_t d = pr->p * (int64_t)(pr->C - 1);
    double *trial = (double *)malloc(sizeof(double) * (size_t)d);
    const double slope = (double)ldot(d, P, g);
    double alpha = 1.0, ft = 0.0;
    int i = 0, evals = 0, good = 0;
    for (;;) {
        for (int64_t t = 0; t < d; ++t) trial[t] = W[t] + alpha * P[t];
        ft = orc_objective(pr, trial);
        ++evals;
        if (!(ft > fW + alpha * beta * slope)) { good = 1; break; }
        if (i > imax) break;
        ++i;
        alpha *= rho;
    }
    free(trial);
    *alpha_out = alpha; *f_new = ft; *ok = good;
    return evals;
}

/*
 * Alg. 1 with a full gradient and a sub-sampled Hessian.  The index sets are
 * inputs: iteration k uses S_all[k*nS .. (k+1)*nS).  W is updated in place.
 * log (optional, 6 doubles per iteration): f(W_k), ||g_k||, CG products, CG
 * relative residual of p_best, step alpha, line-search evaluations (negative
 * if Armijo was not met).  Returns the number of iterations performed.
 */
int orc_ssn(const orc_problem *pr, double *W, int iters, const int32_t *S_all, int64_t nS,
            double eps, double theta, int T, double beta, double rho, int imax, double *log)
{
    const int64_t d = pr->p * (int64_t)(pr->C - 1);
    double *g = (double *)malloc(sizeof(double) * (size_t)d);
    double *dir = (double *)malloc(sizeof(double) * (size_t)d);
    int k = 0;
    for (; k < iters; ++k) {
        double f;
        orc_gradient(pr, W, g, &f);
        const double gn = sqrt((double)ldot(d, g, g));
        if (log) { log[6*k] = f; log[6*k+1] = gn; log[6*k+2] = log[6*k+3] = log[6*k+4] = log[6*k+5] = 0.0; }
        if (gn < eps) break;
        const int32_t *S = S_all + (int64_t)k * nS;
        double rel; int32_t fl;
        const int np = orc_cg(pr, W, S, nS, g, theta, T, dir, &rel, &fl, NULL);
        double alpha, fn; int32_t ok;
        const int ev = orc_linesearch(pr, W, dir, g, f, beta, rho, imax, &alpha, &fn, &ok);
        for (int64_t t = 0; t < d; ++t) W[t] += alpha * dir[t];
        if (log) { log[6*k+2] = np; log[6*k+3] = rel; log[6*k+4] = alpha; log[6*k+5] = ok ? ev : -ev; }
    }
    free(dir); free(g);
    return k;
}

/*
 * Alg. 1 with BOTH the gradient and the Hessian sub-sampled (eqs. (2a), (2b); the paper's
 * "SubsampledNewton-20" uses 20 % of the rows for g and 5 % for H).  Iteration k uses the gradient
 * sample Sg_all[k*nSg ..) and the Hessian sample S_all[k*nS ..).  The Armijo test of Alg. 3 compares
 * the FULL objective F; the paper does not say where F(x_k) comes from when no full gradient pass
 * produces it: here it is evaluated once at the start and afterwards carried over from the accepted
 * line-search trial of the previous iteration (the same number).  log as in orc_ssn, with ||g_k|| the
 * norm of the sub-sampled gradient.
 */
int orc_ssn_sg(const orc_problem *pr, double *W, int iters, const int32_t *Sg_all, int64_t nSg,
               const int32_t *S_all, int64_t nS, double eps, double theta, int T, double beta, double rho,
               int imax, double *log)
{
    const int64_t d = pr->p * (int64_t)(pr->C - 1);
    double *g = (double *)malloc(sizeof(double) * (size_t)d);
    double *dir = (double *)malloc(sizeof(double) * (size_t)d);
    double f = orc_objective(pr, W);
    int k = 0;
    for (; k < iters; ++k) {
        orc_gradient_sampled(pr, W, Sg_all + (int64_t)k * nSg, nSg, g, NULL);
        const double gn = sqrt((double)ldot(d, g, g));
        if (log) { log[6*k] = f; log[6*k+1] = gn; log[6*k+2] = log[6*k+3] = log[6*k+4] = log[6*k+5] = 0.0; }
        if (gn < eps) break;
        const int32_t *S = S_all + (int64_t)k * nS;
        double rel; int32_t fl;
        const int np = orc_cg(pr, W, S, nS, g, theta, T, dir, &rel, &fl, NULL);
        double alpha, fn; int32_t ok;
        const int ev = orc_linesearch(pr, W, dir, g, f, beta, rho, imax, &alpha, &fn, &ok);
        for (int64_t t = 0; t < d; ++t) W[t] += alpha * dir[t];
        f = fn;
        if (log) { log[6*k+2] = np; log[6*k+3] = rel; log[6*k+4] = alpha; log[6*k+5] = ok ? ev : -ev; }
    }
    free(dir); free(g);
    return k;
}

/*
 * Preprocessing of Sec. 4: divide each feature (column) by its 2-norm, so that every non-zero column has length 1; in place.
 * Dense (X != NULL, n-by-p, leading dimension ldx) or CSR (rowptr / colidx / vals).  colnorm (p
 * doubles) receives the norms BEFORE scaling; a column whose norm is zero is left as it is.
 */
void orc_normalize_columns(int64_t n, int64_t p, double *X, int64_t ldx, const int64_t *rowptr,
                           const int32_t *colidx, double *vals, double *colnorm)
{
    long double *ss = (long double *)calloc((size_t)p, sizeof(long double));
    if (X) {
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < p; ++j)
                ss[j] += (long double)X[i * ldx + j] * (long double)X[i * ldx + j];
    } else {
        for (int64_t t = rowptr[0]; t < rowptr[n]; ++t)
            ss[colidx[t]] += (long double)vals[t] * (long double)vals[t];
    }
    for (int64_t j = 0; j < p; ++j)
        colnorm[j] = (double)sqrtl(ss[j]);
    if (X) {
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < p; ++j)
                if (colnorm[j] > 0.0) X[i * ldx + j] /= colnorm[j];
    } else {
        for (int64_t t = rowptr[0]; t < rowptr[n]; ++t)
            if (colnorm[colidx[t]] > 0.0) vals[t] /= colnorm[colidx[t]];
    }
    free(ss);
}
