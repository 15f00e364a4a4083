/*
 * ssn.h -- C ABI of the MI355X (gfx950) sub-sampled Newton hot path for
 * L2-regularised multinomial logistic regression, after "GPU Accelerated
 * Sub-Sampled Newton's Method" (arXiv 1802.09113).
 *
 * Problem (Sec. 3.3, eq. (5)): data matrix A (here X) with n rows and p
 * features, labels b_i in {0..C-1}, weights x = [x_1;...;x_{C-1}] (here the
 * p-by-K matrix W, K = C-1).  Label C-1 is the reference class whose margin is
 * identically zero.
 *
 * Conventions common to every entry point
 *   - Every function returns an int status: SSN_OK (0) or a negative SSN_E_*.
 *     No exception crosses this boundary; ssn_strerror() names a status and
 *     ssn_last_error() returns the context's last detailed message.
 *   - Pointers marked [dev] are DEVICE pointers owned by the caller and only
 *     borrowed: X / CSR arrays / labels for the life of the context, all other
 *     arguments for the duration of the call.  The data must not change while
 *     the context exists: it keeps views derived from them (the column-sorted
 *     entries of a CSR matrix, a padded copy of the last dense row).  Pointers marked [host] are
 *     HOST pointers.  The library owns only the workspace inside ssn_ctx.
 *   - Work is enqueued on the context's stream (a hipStream_t passed as
 *     void*; NULL = the default stream).  Calls that return a scalar through
 *     a [host] pointer return once everything they enqueued has completed
 *     (they wait for the last kernel's result to arrive in host memory, or
 *     for the stream); all other calls are asynchronous.
 *   - Element type T is float (SSN_F32) or double (SSN_F64) for X/vals, W, V,
 *     G, HV, P.  Sums over rows are carried in fp64 in both cases.
 *   - W, V, G, HV, P (direction) are p-by-K, row-major, class index fastest,
 *     leading dimension ldw >= K elements: entry (j,c) at [j*ldw + c].  This
 *     is the paper's vec(.) ordering up to a fixed permutation, so norms and
 *     inner products agree with the paper's d-vector.
 *   - Scaling (SSN_SCALE_MEAN, the default): f and grad f carry 1/n on the
 *     data term and the sampled Hessian 1/|S|.  SSN_SCALE_SUM reproduces the
 *     paper's eq. (1) and (2b): factors 1 and n/|S|.  The regulariser
 *     (lambda/2)||W||^2 is never scaled.
 *   - Dense MFMA kernels handle 2 <= C <= 33 (K <= 32); CSR kernels 2 <= C <= 65.
 */
#ifndef SSN_H
#define SSN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ssn_ctx ssn_ctx;

typedef enum { SSN_F32 = 0, SSN_F64 = 1 } ssn_dtype;
typedef enum { SSN_DENSE_ROWMAJOR = 0, SSN_CSR = 1 } ssn_layout;
typedef enum { SSN_SCALE_MEAN = 0, SSN_SCALE_SUM = 1 } ssn_scale;

enum {
    SSN_OK = 0,
    SSN_E_INVALID_ARG = -1,   /* NULL pointer, size < 1, lambda < 0, ld too small, misaligned ...   */
    SSN_E_BAD_LABEL = -2,     /* a label outside [0,C)                                           */
    SSN_E_BAD_INDEX = -3,     /* a sample index outside [0,n) or a CSR column outside [0,p)      */
    SSN_E_NOT_PREPARED = -4,  /* ssn_hess_apply / ssn_cg before ssn_hess_prepare                 */
    SSN_E_ALLOC = -5,         /* device allocation failed                                        */
    SSN_E_HIP = -6,           /* a HIP runtime call failed                                       */
    SSN_E_NONFINITE = -7,     /* objective evaluated to NaN/Inf                                  */
    SSN_E_UNSUPPORTED = -8,   /* shape outside the supported range (e.g. C too large)            */
    SSN_E_TOO_LARGE = -9      /* ssn_hessvec_static: the problem needs more than the fixed workspace */
};

/* Problem description.  Copied by ssn_create; the arrays it points to are borrowed. */
typedef struct {
    int64_t n, p;             /* rows, features                                                  */
    int32_t C;                /* classes (K = C-1 weight columns)                                */
    int32_t dtype;            /* ssn_dtype                                                       */
    int32_t layout;           /* ssn_layout                                                      */
    int32_t scale;            /* ssn_scale                                                       */
    double lambda;            /* L2 regularisation, >= 0                                         */
    const void *X;            /* [dev] dense: n-by-p row-major, element (i,j) at [i*ldx + j];    */
    int64_t ldx;              /*       leading dimension in elements, >= p; storage of n*ldx     */
                              /*       elements, or (n-1)*ldx + p when ldx == p                  */
    const int32_t *rowptr;    /* [dev] CSR: n+1 offsets                                          */
    const int32_t *colidx;    /* [dev] CSR: nnz column ids in [0,p), ascending inside a row      */
    const void *vals;         /* [dev] CSR: nnz values of type T                                 */
    int64_t nnz;              /*       CSR: number of stored entries (< 2^31)                    */
    const int32_t *labels;    /* [dev] n labels in [0,C)                                         */
    int64_t ldw;              /* leading dimension of W, V, G, HV, P in elements, >= K           */
    void *stream;             /* hipStream_t, or NULL                                            */
} ssn_desc;

/* Result of ssn_cg (Alg. 2). */
typedef struct {
    int32_t iters;            /* Hessian-vector products made (<= T)                             */
    int32_t flags;            /* bit0: stopped by ||r|| <= theta ||g||; bit1: s^T H s <= 0 met   */
    double rel_res;           /* ||r_best|| / ||g||                                              */
    double gnorm;             /* ||g||                                                           */
} ssn_cg_info;

/* ssn_params.flags.  By default ssn_solve evaluates the first line-search trial (alpha = 1) with the
 * gradient pass, which returns F and grad F from one read of the data; when that trial is accepted -- the
 * usual case for a Newton-type step -- the trial point is the next iterate and its gradient is already
 * there, so the iteration costs one pass over the data less.  The iterates, F values and step lengths are
 * those of Alg. 1 and Alg. 3 either way (the two passes add the same row terms in a different order, so F
 * may differ in the last bits); only the phase times move: the gradient's time is then reported inside
 * ms_linesearch of the previous iteration.  After a rejected first trial the plain objective pass is used
 * until a first trial is accepted again.  Not used with a sub-sampled gradient.  This flag turns it off. */
#define SSN_SOLVE_NO_LOOKAHEAD 1
/* Leave out the six stream events per iteration behind the ms_* fields of the iteration records (which then
 * hold NaN): each record costs a few microseconds of device time. */
#define SSN_SOLVE_NO_PHASE_TIMES 2
/* Back-tracking trials of the line search (every trial after the first) are evaluated on cached margins:
 * X (W + alpha P) = X W + alpha X P, so one pass over the data leaves X W and X P (n rows of 2K numbers) and each
 * further trial is a pass over those instead of over X.  The same F up to rounding; Alg. 3's trial sequence and
 * exit rules are unchanged.  This flag makes every trial a pass over the data, as Alg. 3 is written. */
#define SSN_SOLVE_NO_MARGIN_CACHE 4

/* Parameters of ssn_solve (Alg. 1, 2, 3).  The paper gives no numeric values for beta, rho,
 * i_max; textbook values are the defaults chosen by callers. */
typedef struct {
    int32_t iters;            /* SSN iterations to run (the paper ran a fixed count)             */
    int32_t T;                /* max CG products per iteration                                   */
    int32_t imax;             /* line search: give up after more than imax step reductions       */
    int32_t flags;            /* 0, or SSN_SOLVE_NO_LOOKAHEAD | SSN_SOLVE_NO_PHASE_TIMES         */
    int64_t nS;               /* Hessian sample size per iteration                               */
    double eps;               /* stop when ||g|| < eps                                           */
    double theta;             /* CG relative residual tolerance                                  */
    double beta;              /* Armijo constant                                                 */
    double rho;               /* back-tracking factor                                            */
    const int32_t *S_all;     /* [dev] iters*nS sample indices, iteration k uses [k*nS,(k+1)*nS) */
    ssn_ctx *test;            /* optional context holding held-out rows: accuracy per iteration  */
    const int32_t *Sg_all;    /* [dev, nullable] iters*nSg gradient sample indices (eq. (2a)): iteration
                                 k forms g on [k*nSg,(k+1)*nSg); NULL = full gradient of eq. (6)     */
    int64_t nSg;              /* gradient sample size (ignored when Sg_all is NULL)                */
} ssn_params;

/* One record per SSN iteration, written by ssn_solve to a [host] array. */
typedef struct {
    double f;                 /* objective at the iterate the iteration started from             */
    double gnorm;             /* ||grad f|| there                                                */
    double cg_rel_res;        /* relative residual of the direction taken                        */
    double alpha;             /* step length                                                     */
    double test_acc;          /* accuracy on params.test after the update (NaN if none)          */
    double ms_grad, ms_prepare, ms_cg, ms_linesearch, ms_update;   /* device time per phase, from
                                 stream events (NaN with SSN_SOLVE_NO_PHASE_TIMES)                */
    int32_t cg_iters;         /* Hessian-vector products                                         */
    int32_t ls_evals;         /* objective evaluations in the line search                        */
    int32_t ls_ok;            /* 1 iff the Armijo condition held at the returned step            */
    int32_t reserved;
} ssn_iter_record;

const char *ssn_strerror(int status);
const char *ssn_last_error(const ssn_ctx *ctx);

/* Preprocessing of Sec. 4 (unit column norms), in place on the
 * device, before ssn_create: dense X [dev] n-by-p with leading dimension ldx, or CSR rowptr / colidx /
 * vals [dev] with nnz stored entries (the other layout's pointers are ignored).  colnorm [dev, p doubles]
 * receives the column norms before scaling; a column of norm zero is left as it is.  Column indices of a
 * CSR matrix must lie in [0,p) (not checked here; ssn_create checks them).  Sums in a fixed order.
 * Allocates temporaries, synchronises the stream.  Returns SSN_OK, SSN_E_INVALID_ARG, SSN_E_ALLOC or
 * SSN_E_HIP. */
int ssn_normalize_columns(int32_t layout, int32_t dtype, int64_t n, int64_t p, void *X, int64_t ldx,
                          const int32_t *rowptr, const int32_t *colidx, void *vals, int64_t nnz, double *colnorm,
                          void *stream);

/* Create a context for one data set.  Validates the description (C >= 2, n,p >= 1, lambda >= 0,
 * ldx >= p, ldw >= K, labels in range, CSR columns in range; one device pass over labels / CSR
 * indices) and allocates the workspace.  Synchronises the stream. */
int ssn_create(ssn_ctx **out, const ssn_desc *desc);
int ssn_destroy(ssn_ctx *ctx);
int ssn_set_stream(ssn_ctx *ctx, void *stream);

/* Objective, eq. (5) with the stable log-sum-exp of eq. (8), (9) and the four-part form of
 * Alg. 5 / eqs. (14)-(17):
 *   f = s * sum_i [ M_i + log(alpha_i) - sum_c 1(b_i = c) z_ic ] + (lambda/2) ||W||_F^2 ,  z_i = W^T x_i.
 * W [dev] p-by-K; f [host].  One pass over X. */
int ssn_objective(ssn_ctx *ctx, const void *W, double *f);

/* Gradient, eq. (6) / Alg. 6:  G = s * X^T (P - Y) + lambda W, P the row-wise class
 * probabilities, Y the one-hot labels without the reference class.
 * W [dev], G [dev] p-by-K out; f [host], may be NULL -- if given, also receives f(W) from the
 * same pass and the call synchronises. */
int ssn_gradient(ssn_ctx *ctx, const void *W, void *G, double *f);

/* The same two calls with the scalar left on the device (the function-pointer style F(.) of Alg. 2 / Alg. 3
 * for callers that keep their control flow on the device, and the problem statement of Sec. 3.3 otherwise
 * unchanged): f_dev [dev] receives f(W); kernels are enqueued only, nothing is read back and the host does
 * not wait, so the call may be recorded into a HIP graph on the context's stream (dense layouts; the first
 * gradient on a CSR context builds its column-sorted view and waits for the stream once).  A non-finite
 * value is stored as it is (no SSN_E_NONFINITE). */
int ssn_objective_dev(ssn_ctx *ctx, const void *W, double *f_dev);
int ssn_gradient_dev(ssn_ctx *ctx, const void *W, void *G, double *f_dev);

/* Sub-sampled gradient, eq. (2a), on the index multiset S [dev] (nS entries in [0,n), repeats allowed):
 *   G = s_S * X_S^T (P_S - Y_S) + lambda W,  s_S = 1/nS (mean scaling) or n/nS (sum scaling).
 * Same kernels as ssn_gradient on the sampled rows.  f_S [host, nullable] receives the objective of the
 * same sample, s_S * sum_{i in S} f_i(W) + (lambda/2)||W||^2 (then the call synchronises).  Validates S. */
int ssn_gradient_sampled(ssn_ctx *ctx, const void *W, const int32_t *S, int64_t nS, void *G, double *f_S);

/* Sub-sampled Hessian (eq. (2b)) at W on the index multiset S [dev] (nS entries in [0,n),
 * repeats allowed, any order): computes and caches the probabilities of the sampled rows (the
 * matrix W of eq. (11); it depends on the weights only, so all CG products of one SSN
 * iteration reuse it).  S is borrowed until the next prepare.  Validates S. */
int ssn_hess_prepare(ssn_ctx *ctx, const void *W, const int32_t *S, int64_t nS);

/* Hessian-vector product, eqs. (10)-(13) / Alg. 7, 8 on the prepared sample:
 *   HV = s_S * X_S^T U + lambda V,  U_i = (diag(p_i) - p_i p_i^T)(V^T x_i).
 * V [dev] in, HV [dev] out (must not alias V).  Enqueues kernels only: no allocation, no wait for the
 * device, so the call may be recorded into a HIP graph on the context's stream (so may ssn_gradient with
 * f == NULL on a dense matrix, and ssn_axpy). */
int ssn_hess_apply(ssn_ctx *ctx, const void *V, void *HV);

/* ssn_hess_prepare followed by ssn_hess_apply. */
int ssn_hessvec(ssn_ctx *ctx, const void *W, const int32_t *S, int64_t nS, const void *V, void *HV);

/* Conjugate gradient with best-iterate memory, Alg. 2, on H_S p = -g for the prepared H_S.
 * G [dev] right-hand side gradient; P_out [dev] receives p_best; at most T products.
 * trace [host, nullable, 3*T doubles]: per product k the step alpha_k, ||r_{k+1}||, s_k^T H s_k.
 * The whole loop runs on the device without host round trips; the call synchronises once at
 * the end to fill info / trace.  The iterates are those of Alg. 2 up to rounding; how they are formed:
 *   - No inner product waits for a vector: with Z = X_S v and U the rows of eq. (12), v^T (X_S^T U) is the
 *     sum over the sample of z_i . u_i, which the product's own launch leaves as partial sums.
 *   - Dense layouts: the product is applied to the residual r_k (H is linear, so with line 12
 *     H s_k = H r_k + beta H s_{k-1}; H s is kept as a vector and updated), and
 *     s_k^T H s_k = r_k^T H r_k + 2 beta r_k^T H s_{k-1} + beta^2 s_{k-1}^T H s_{k-1}: two launches per product.
 *     The theta test for r_k is made after product k has been enqueued, so a run that stops early has made
 *     one product more than info.iters reports (its result is discarded).
 *   - CSR layout: H_S acts as lambda I on every coordinate whose column no sampled row touches, so r, s, p
 *     stay multiples of g there; the vectors of Alg. 2 are kept on the sampled columns only, three scalars
 *     carry the rest, and P_out is assembled at the end. */
int ssn_cg(ssn_ctx *ctx, const void *G, double theta, int32_t T, void *P_out,
           ssn_cg_info *info, double *trace);

/* Back-tracking line search, Alg. 3 / eq. (3c): alpha = 1; while f(W + alpha P) > fW +
 * alpha*beta*<P,G>: if i > imax stop; i++; alpha *= rho.
 * W, P, G [dev]; alpha, f_new, n_eval, ok [host] outputs (ok = 1 iff Armijo held at exit).
 * The trials are evaluated on cached margins (one pass over the data for X W and X P, then n*2K numbers per
 * trial; see SSN_SOLVE_NO_MARGIN_CACHE), except on dense matrices with more than 16 weight columns.  The first
 * call allocates the cache (n * 2K elements). */
int ssn_linesearch(ssn_ctx *ctx, const void *W, const void *P, const void *G, double fW,
                   double beta, double rho, int32_t imax,
                   double *alpha, double *f_new, int32_t *n_eval, int32_t *ok);

/* Classification rule (end of Sec. 3.3): argmax over [z_0..z_{K-1}, 0], ties to the lowest
 * class index.  pred [dev, nullable] n int32; acc [host, nullable] = mean(pred == labels). */
int ssn_predict(ssn_ctx *ctx, const void *W, int32_t *pred, double *acc);

/* Accuracy of the classification rule (end of Sec. 3.3) on held-out rows: test [host] describes them like
 * an ssn_desc for ssn_create (X or CSR arrays and labels [dev]; n of its own; p, C, dtype and ldw equal to the
 * context's; lambda, scale and stream are ignored).  acc [host] = mean(argmax == label).  Validates the
 * description like ssn_create, allocates a temporary workspace and synchronises the stream; callers that
 * evaluate the same held-out rows many times keep a second context and call ssn_predict on it instead
 * (ssn_params.test does that inside ssn_solve). */
int ssn_accuracy(ssn_ctx *ctx, const ssn_desc *test, const void *W, double *acc);

/* The paper stacks the K weight columns into one d-vector, x = [x_1; ...; x_K] (Sec. 3.3, eq. (5)): element
 * c*p + j of vec is element (j, c) of the p-by-K block used everywhere in this library.  These two calls
 * convert between the orderings on the device (vec [dev]: p*K elements of type T; block [dev]: p-by-K with
 * leading dimension ldw; the two must not overlap).  Asynchronous. */
int ssn_vec_to_rowmajor(ssn_ctx *ctx, const void *vec, void *block);
int ssn_rowmajor_to_vec(ssn_ctx *ctx, const void *block, void *vec);

/* Sub-sampled Newton, Alg. 1 with the full gradient and a sampled Hessian:
 * per iteration f,g at W; stop if ||g|| < eps; prepare H_S; CG; line search; W += alpha P.
 * With params.Sg_all the gradient is the sub-sampled one of eq. (2a); the Armijo test still compares the
 * full objective, evaluated once at the start and then carried over from the accepted trial.
 * W_inout [dev]; log [host, nullable] receives min(iterations, max_log) records;
 * iters_done [host, nullable]. */
int ssn_solve(ssn_ctx *ctx, void *W_inout, const ssn_params *params,
              ssn_iter_record *log, int32_t max_log, int32_t *iters_done);

/* y = a*x + y style helper used by callers that drive Alg. 1 themselves: W += alpha * P. */
int ssn_axpy(ssn_ctx *ctx, double alpha, const void *P, void *W_inout);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the product of ssn_hessvec on a dense matrix without a context and
 * without any allocation.  d [host] describes the data as for ssn_create (layout SSN_DENSE_ROWMAJOR only);
 * W, V [dev] in, HV [dev] out (p-by-K, leading dimension d->ldw, HV must not alias V or W); S [dev] nS
 * indices in [0, d->n), repeats allowed.  The probabilities of the sampled rows, the per-workgroup partial
 * sums and a padded copy of the last row live in a fixed workspace of SSN_STATIC_WORKSPACE_BYTES inside the
 * library's device image (one copy per GPU, held until the process ends): a problem that needs more returns
 * SSN_E_TOO_LARGE, CSR or K > 32 SSN_E_UNSUPPORTED, a bad description SSN_E_INVALID_ARG, a failed launch
 * SSN_E_HIP.  Nothing is validated on the device: labels are not read, and the indices in S are the
 * caller's responsibility (ssn_hessvec checks them).  Kernels are enqueued on d->stream and the call returns
 * without waiting.  Every call on a GPU uses that GPU's one workspace, so two calls whose kernels may
 * overlap on the same GPU (different streams, or threads) race; calls on one stream are safe. */
#define SSN_STATIC_WORKSPACE_BYTES (48u << 20)
int ssn_hessvec_static(const ssn_desc *d, const void *W, const int32_t *S, int64_t nS, const void *V, void *HV);

#ifdef __cplusplus
}
#endif
#endif /* SSN_H */
