// Internal declarations shared by the translation units of libssn_hip.so.
// Nothing here is part of the public C ABI (that is include/ssn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>

#include "ssn.h"

namespace ssn {

struct CgSlot;

// ---- per-row epilogue selector of the row-block kernels -------------------------------
enum RowMode : int {
    ROW_OBJ = 0,    // loss only                                   (Alg. 5)
    ROW_GRAD = 1,   // loss + U = P - Y                            (Alg. 6)
    ROW_PREP = 2,   // store P                                     (eq. (11))
    ROW_APPLY = 3,  // U = P .* Vhat - P .* ((P .* Vhat) e e^T)    (eq. (12), Alg. 8)
    ROW_PRED = 4,   // argmax classification + hit count
    ROW_MARGIN = 5  // store the margins of two operands, Z = [X M | X M2] (row stride KP): the line search's cache
};

// Arguments of the "rows" kernels: Z = X_rows * M followed by a per-row epilogue.
struct RowsArgs {
    // data (dense or CSR)
    const void *X;
    int64_t ldx;
    const int32_t *rowptr, *colidx;
    const void *vals;
    int64_t n, p;
    int32_t K;
    const int32_t *labels;
    // which rows: S == nullptr -> rows 0..nrows-1, else rows S[0..nrows-1]
    const int32_t *S;
    int64_t nrows;
    // right operand, p x K, leading dimension ldm
    const void *M;
    int64_t ldm;
    const void *M2;      // ROW_MARGIN: second right operand (same leading dimension)
    // per-row buffers with row stride KP (padded K): Pin read by ROW_APPLY, UP written by GRAD/PREP/APPLY
    const void *Pin;
    void *UP;
    int32_t KP;
    // outputs
    double *loss_part;   // one partial per wave (OBJ, GRAD)
    int32_t *pred;       // nullable (PRED)
    int32_t *hit_part;   // one partial per wave (PRED)
    int32_t mode;
    const int32_t *skip; // nullable device flag: non-zero -> the launch does nothing
    void *part;          // one-pass kernel only: per-workgroup p x K partial sums of X^T U
    int32_t fw;          // one-pass kernel only: features per wave (set by the launcher)
    // one-pass kernel only: zero-padded copy of row n-1, tail_len elements = what the kernel may read from the
    // start of a row (max(ldx, p rounded up to the vector width), capped where no lane reaches): it reads whole
    // vectors, which on every other row stay inside the row's storage or reach into the next row
    const void *tail_row;
    int32_t tail_len;
    // CSR rows kernel only: non-zero -> a workgroup per row, the row's entries shared out among its four waves (set by
    // the launcher for passes over few, long rows)
    int32_t csr_split;
    // CSR, one weight column, full passes only (set by the launcher): the row that holds entry 64 w for every aligned
    // window of 64 stored entries, the rows' margins (n values), the windows' leading partial sums, the entry count
    const int32_t *rwin;
    void *zrow, *zhead;
    int64_t nnz;
};

// Arguments of the transposed product: part[chunk] = X_rows(chunk)^T * U(chunk).
struct XtuArgs {
    const void *X;
    int64_t ldx;
    const int32_t *rowptr, *colidx;
    const void *vals;
    int64_t n, p;
    int32_t K;
    const int32_t *S;
    int64_t nrows;
    const void *U;       // nrows_pad x KP
    int32_t KP;
    void *part;          // nchunks x p x K (element type T)
    int64_t rows_per_chunk;
    int32_t nchunks;
    const int32_t *skip;
    // Sampled product on few row blocks of a wide matrix: U is not read but formed here, eq. (12), from the partial
    // margins of `nslices` feature slices (Zpart[s][row][16], zrows rows per slice) and the probabilities Pin (row
    // stride KP); the chunk's sum of z_i . u_i goes to zu_part[chunk].  Zpart == nullptr: U is read.
    const void *Zpart;
    int32_t nslices;
    int64_t zrows;
    const void *Pin;
    double *zu_part;
};

// out = scale * sum_chunks part + lambda * M ; optional per-block partials of <out, M>.
struct FinArgs {
    const void *part;
    int32_t nchunks;
    int64_t p;
    int32_t K;
    double scale, lambda;
    const void *M;
    int64_t ldm;
    void *out;
    int64_t ldo;
    double *dot_part;    // nullable; FIN_BLOCKS entries
    const int32_t *skip;
};

constexpr int ROWS_WAVES_PER_BLOCK = 4;
constexpr int RED_MAX_PARTS = 1024;   // upper bound on partial-sum arrays consumed by single-block reducers
constexpr int VEC_BLOCK = 256;

// grid sizes: blocks of the rows kernels (4 wave partials each), of the level-1 kernels (one partial
// each, <= RED_MAX_PARTS) and of the finalize kernel (one <.,.> partial each, <= RED_MAX_PARTS)
int rows_grid_blocks(int64_t nrows, int num_cus);
int vec_blocks(int64_t total);
int finalize_blocks(int64_t p, int K);

// ---- launchers (dense_mfma.hip / csr.hip / vecops.hip) ---------------------------------
void dense_rows_plan(int dtype, int64_t nrows, int64_t p, int K, int num_cus, int *blocks, int *split_waves);
hipError_t launch_dense_rows(int dtype, const RowsArgs &a, int blocks, int split_waves, hipStream_t st);
hipError_t launch_dense_xtu(int dtype, const XtuArgs &a, hipStream_t st);
// partial margins of feature slices: Zpart[s][row][16] = X_rows[:, slice s] * M[slice s, :] for `nslices` slices of
// `fper` features (a multiple of 32), a workgroup of eight waves per (row block, slice); K <= 16, 16-byte aligned rows
// rwin[w] = the row that holds stored entry 64 w (w < ceil(nnz / 64)); rows may be empty
hipError_t launch_csr_window_rows(const int32_t *rowptr, int64_t n, int64_t nnz, int32_t *rwin, hipStream_t st);
hipError_t launch_dense_zpart(int dtype, const RowsArgs &a, void *Zpart, int nslices, int64_t fper, hipStream_t st);
bool dense_fused_supported(int dtype, const RowsArgs &a);
int dense_fused_grid(int dtype, const RowsArgs &a, int num_cus);
int dense_fused_waves(int dtype, const RowsArgs &a);
hipError_t launch_dense_fused(int dtype, const RowsArgs &a, int grid, hipStream_t st);
// long passes over narrow matrices on the vector units (dense_narrow.hip); the three calls above route to it when
// it applies, with the same contract: `grid` partials in a.part, 4 * `grid` loss partials
bool dense_narrow_applies(int dtype, const RowsArgs &a);
int dense_narrow_grid(int dtype, const RowsArgs &a, int num_cus);
int dense_narrow_max_grid(int64_t p, int num_cus);       // 0: no narrow launch on matrices of p features
hipError_t launch_dense_narrow(int dtype, const RowsArgs &a, int grid, hipStream_t st);
hipError_t launch_csr_rows(int dtype, const RowsArgs &a, int blocks, hipStream_t st);
// binary problem (K = 1) on a dense matrix: matrix-vector kernels on the vector units (dense_binary.hip)
int binary_rows_blocks(int64_t nrows, int num_cus);
hipError_t launch_binary_rows(int dtype, const RowsArgs &a, int blocks, hipStream_t st);
hipError_t launch_binary_xtu(int dtype, const XtuArgs &a, hipStream_t st);
hipError_t launch_finalize(int dtype, const FinArgs &a, int blocks, hipStream_t st);

// out = lambda * M (p x K), with optional <.,.> partials disabled; used by the CSR path before scattering
hipError_t launch_scale_copy(int dtype, int64_t p, int K, double lambda, const void *M, int64_t ldm,
                             void *out, int64_t ldo, const int32_t *skip, hipStream_t st);

// partials of <A, B> over the p x K block: part[b] for b < blocks
hipError_t launch_dot_part(int dtype, int64_t p, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
                           double *part, int blocks, const int32_t *skip, hipStream_t st);
// to_block: block (p x K row-major, leading dimension ld) <- vec (class-major d-vector, element c * p + j);
// otherwise vec <- block
hipError_t launch_vec_layout(int dtype, int64_t p, int K, void *vec, void *block, int64_t ld, bool to_block,
                             hipStream_t st);
// dst[0..len) = src[0..n) followed by zeros
hipError_t launch_pad_copy(int dtype, const void *src, int64_t n, void *dst, int64_t len, hipStream_t st);
// Y = alpha * X + Z (Y may alias Z)
hipError_t launch_axpy(int dtype, int64_t p, int K, double alpha, const void *X, int64_t ldx_,
                       const void *Z, int64_t ldz, void *Y, int64_t ldy, hipStream_t st);
// Y = alpha X + Z with one partial of ||Y||^2 per block (blocks <= RED_MAX_PARTS)
hipError_t launch_axpy_sq(int dtype, int64_t p, int K, double alpha, const void *X, int64_t ldx, const void *Z, int64_t ldz,
                          void *Y, int64_t ldy, double *sq_part, int blocks, hipStream_t st);
// partials of A.A, A.B, B.B (blocks entries each, one after the other) from one pass over the two p x K blocks
hipError_t launch_dot3_part(int dtype, int64_t p, int K, const void *A, int64_t lda, const void *B, int64_t ldb, double *part,
                            int blocks, hipStream_t st);
// Line search on cached margins (Alg. 3 with X (W + alpha P) = X W + alpha X P): Z holds n rows [X W | X P] of 2K
// values (row stride kp); one loss partial per block for the trial step alpha
hipError_t launch_ls_trial(int dtype, const void *Z, int kp, int64_t n, int K, const int32_t *labels, double alpha,
                           double *loss_part, int blocks, hipStream_t st);
// *out (and the host-visible word, then the ticket) = scale * sum(loss) + half_lambda * (ww + 2 alpha wp + alpha^2 pp)
// with ww, wp, pp the sums of three partial arrays of nd entries each (dots[0..nd), [nd..2nd), [2nd..3nd))
hipError_t launch_ls_value(const double *loss_part, int nparts, double scale, const double *dots, int nd, double alpha,
                           double half_lambda, double *out, double *out_host, unsigned long long *ticket_host,
                           unsigned long long ticket, hipStream_t st);
// *out = scale * sum(a[0..na)) + coef * sum(b[0..nb))   (single block, fixed order)
// *out (and *out_host, nullable, host-visible) = scale * sum(loss_part) + half_lambda * ||W||_F^2 ; one block, for
// blocks of up to OBJ_VALUE_ELEMS elements
hipError_t launch_objective_value(int dtype, const double *loss_part, int nparts, double scale, const void *W, int64_t p,
                                  int K, int64_t ldw, double half_lambda, double *out, double *out_host,
                                  unsigned long long *ticket_host, unsigned long long ticket, hipStream_t st);
constexpr int64_t OBJ_VALUE_ELEMS = 32768;
// out_host / ticket_host (nullable): also post the value to host-visible memory, then the ticket (see post_to_host)
hipError_t launch_combine(const double *a, int na, double scale, const double *b, int nb, double coef, double *out,
                          hipStream_t st, double *out_host = nullptr, unsigned long long *ticket_host = nullptr,
                          unsigned long long ticket = 0);
hipError_t launch_solve_publish(const double *slope_part, int n, const double *f_dev, const CgSlot *fin, double *slope_dev,
                                double *host_out, bool support_only, hipStream_t st);
// streaming read of `bytes` (multiple of 16, 16-byte aligned); one checksum partial per block
hipError_t launch_stream_read(const void *src, int64_t bytes, double *part, int blocks, hipStream_t st);
hipError_t launch_sum_int(const int32_t *a, int na, int32_t *out, hipStream_t st);

// validation passes: *bad receives the number of offending entries
hipError_t launch_check_range(const int32_t *v, int64_t count, int64_t lo, int64_t hi, int32_t *bad, hipStream_t st);
hipError_t launch_check_rowptr(const int32_t *rowptr, int64_t n, int64_t nnz, int32_t *bad, hipStream_t st);

// ---- column-sorted view of a set of CSR rows (csc.hip) --------------------------------------------
struct CscView {
    int64_t nnz = 0;                 // entries in the view
    int32_t npieces = 0;
    int32_t *key = nullptr;          // column of entry t, ascending
    int32_t *row = nullptr;          // position of entry t's row in the row selection the view was built from
    void *val = nullptr;
    int32_t *piece_start = nullptr;  // npieces + 1
    int32_t *piece_col = nullptr;    // npieces + 4 (sentinels -1)
    int64_t nrows = 0;               // rows selected
    void *piece_part = nullptr;      // 2 x npieces x K: partial sums of the pieces of multi-piece columns, then of runs of them
    // construction scratch (kept by the sample view, which is rebuilt at every ssn_hess_prepare)
    int32_t *off = nullptr, *key_in = nullptr, *idx_in = nullptr, *idx_out = nullptr, *row_in = nullptr;
    void *val_in = nullptr;
    int32_t *flag = nullptr, *pid = nullptr;
    void *cub_tmp = nullptr;
    size_t cub_bytes = 0;
    int32_t *count_dev = nullptr;
    int64_t cap = 0, cap_row = 0, cap_val = 0, cap_piece = 0, cap_pcol = 0, cap_part = 0, cap_off = 0, cap_in = 0,
            cap_flag = 0, cap_pid = 0;
    // support of the view (csc_build with support = true): the ncols distinct columns in ascending order, the
    // selected rows as a CSR matrix in those coordinates -- row pointers `off`, column positions `ccol`, values
    // `val_in`, all in the row order of the selection -- and the pieces' column positions
    bool has_support = false;
    int32_t ncols = 0;
    int32_t *cols = nullptr;         // ncols
    int32_t *ccol = nullptr;         // nnz
    int32_t *piece_cpos = nullptr;   // npieces + 4 (sentinels -1)
    int64_t cap_cols = 0, cap_ccol = 0, cap_pcpos = 0, cap_valin = 0;
    // scratch of csc_build_filtered: sample multiplicity of every row of the matrix, bitmap of the sampled rows, the
    // rows' lists of sample positions (head per row, next per sample position), tile sums and offsets of the prefix
    // sums, row lengths of the sample, every sorted entry's place in row order
    int32_t *cnt = nullptr, *head = nullptr, *next = nullptr, *tsum = nullptr, *toff = nullptr, *ftoff = nullptr, *len = nullptr,
            *bitmap = nullptr, *eidx = nullptr;
    int64_t cap_cnt = 0, cap_head = 0, cap_next = 0, cap_tsum = 0, cap_toff = 0, cap_ftoff = 0, cap_len = 0, cap_bitmap = 0,
            cap_eidx = 0;
    // the view of all rows only: place of entry t in the CSR arrays (kept for csc_build_filtered)
    int32_t *csr_pos = nullptr;
    // one weight column: the piece that starts at every aligned 64th entry (csc_window_index, after every build);
    // win_npieces: the piece count it was made for
    int32_t *win_pid = nullptr;
    int64_t cap_win = 0;
    int32_t win_npieces = -1;
};
hipError_t csc_build(CscView *v, int dtype, const int32_t *rowptr, const int32_t *colidx, const void *vals,
                     const int32_t *S, int64_t nrows, int64_t p, int K, hipStream_t st, bool support = false);
// the same view for a sample S[0..nS) of the n rows, filtered out of `full` (the view of all rows) without a sort;
// hipErrorNotSupported: the row lengths are too uneven for its buffer bound, use csc_build
hipError_t csc_build_filtered(CscView *v, const CscView &full, int dtype, const int32_t *rowptr, const int32_t *colidx,
                              const void *vals, const int32_t *S, int64_t nS, int64_t n, int32_t max_len, int K,
                              hipStream_t st, bool support);
// longest row of a CSR matrix (synchronises the stream)
hipError_t csr_max_row_len(const int32_t *rowptr, int64_t n, int32_t *scratch_dev, int32_t *out, hipStream_t st);
// one weight column: index of the view's 64-entry windows for the lane-per-entry product kernel (call after a build)
hipError_t csc_window_index(CscView *v, hipStream_t st);
void csc_free(CscView *v);
void csc_free_scratch(CscView *v);
// out += coef * X_view^T U (U rows indexed like the view's row selection); slot (nullable): multiply by
// -slot->alpha and do nothing once that CG loop has ended
// support_coords: `out` has one row per distinct column of the view (ncols rows) instead of one per column
hipError_t launch_csc_apply(int dtype, const CscView &v, int K, int KP, const void *U, double coef, void *out, int64_t ldo,
                            const CgSlot *slot, const int32_t *skip, hipStream_t st, bool support_coords = false);

// ---- unit-column-norm preprocessing (preprocess.hip); synchronises the stream ------------------------
hipError_t normalize_columns(int layout, int dtype, int64_t n, int64_t p, void *X, int64_t ldx, const int32_t *rowptr,
                             const int32_t *colidx, void *vals, int64_t nnz, double *colnorm, hipStream_t st);

// ---- device-resident CG (Alg. 2) ---------------------------------------------------------
struct CgSlot {          // state before product k
    double rr;           // r_k^T r_k
    double rbest;        // ||r_best||
    double gnorm;        // ||g||
    int32_t done;        // loop has ended (theta test, breakdown, zero gradient)
    int32_t iters;       // products made so far
    int32_t flags;
    int32_t brk;         // set during product k when s^T H s <= 0
    double alpha;        // step length of product k, where a kernel of its own computes it (CSR path)
    int32_t best_cur;    // CSR path: the best iterate is the CURRENT p and has not been copied to p_best yet
    int32_t best_pending;// dense paths: r_k was the best so far, p_best <- p_k is still to be done (by the next pass over p)
    double sHs;          // dense paths: curvature s_k^T H s_k of product k (written with alpha by that product's finalize)
    // CSR path: the CG vectors are kept on the columns the sample touches only.  On every other coordinate j
    // H_S is lambda I, so r_j, s_j, p_j stay multiples of g_j; the multipliers and the sum of g_j^2 over those
    // coordinates (goff; 0 on the dense paths, where the terms below vanish) are all that is needed of them.
    double goff;
    double rho, sigma, pi, pibest;   // r_j = rho g_j, s_j = sigma g_j, p_j = pi g_j, p_best_j = pibest g_j
};

struct CgVecs {
    int64_t p;
    int32_t K;
    int64_t ld;          // leading dimension of every vector below
    const void *G;
    void *pv, *r, *s, *pbest;
};

// ss_part (nullable) receives the same partials again: s_0 = -g
hipError_t launch_cg_init(int dtype, const CgVecs &v, double *gg_part, double *ss_part, int blocks, hipStream_t st);
// gg_full_part (nullable): partials of g.g over ALL coordinates when gg_part covers the sample's columns only
hipError_t launch_cg_init_state(const double *gg_part, int nparts, CgSlot *slot0, hipStream_t st,
                                const double *gg_full_part = nullptr, int n_full = 0);
// CG on the support of the sample: the vectors of v (ld = K, v.p = ncols rows) start from the rows cols[] of G
hipError_t launch_cg_init_support(int dtype, const CgVecs &v, const void *G, int64_t ldg, const int32_t *cols,
                                  double *gg_part, double *ss_part, int blocks, hipStream_t st);
// P_out = fin->pibest * G everywhere, then rows cols[] of it = the rows of pb (ncols x K, ld = K)
// dot_part (nullable): partials of <pb, rows cols[] of G>, *n_dot of them (<= RED_MAX_PARTS)
hipError_t launch_cg_expand(int dtype, int64_t p, int K, const void *G, int64_t ldg, void *P_out, int64_t ldp,
                            const CgSlot *fin, const void *pb, const int32_t *cols, int64_t ncols, double *dot_part,
                            int *n_dot, hipStream_t st);
// CSR path, lines 10-12 (the dense paths do all of lines 7-12 in finalize_cg_kernel).  ss_part (nullable): one partial
// of s.s per block for the new direction; update_p: also p += cur->alpha * s, and p_best is then kept lazily
// (CgSlot::best_cur): launch_cg_finish after the last product completes it; lambda: for the off-support scalars
hipError_t launch_cg_step2(int dtype, const CgVecs &v, const CgSlot *cur, CgSlot *next, const double *rr_part,
                           int n_rr, double theta, double *trace_k, double *ss_part, bool update_p, int blocks,
                           hipStream_t st, double lambda = 0.0);
// CSR path, lines 7-9 in pieces: cur->alpha from the partials of sum_i z_i . u_i and of s.s (one block); then the
// sparse part of r -= alpha H s goes through the column-sorted gather (launch_csc_apply) and the rest,
// r -= alpha lambda s with the partials of the new r.r, through launch_cg_r_update
// p_best = p where the final state says the best iterate is still only in p
hipError_t launch_cg_finish(int dtype, const CgVecs &v, const CgSlot *fin, int blocks, hipStream_t st);
hipError_t launch_cg_alpha(CgSlot *cur, const double *zu_part, int n_zu, const double *ss_part, int n_ss, double scale,
                           double lambda, double *trace_k, hipStream_t st);
hipError_t launch_cg_r_update(int dtype, const CgVecs &v, const CgSlot *cur, double lambda, double *rr_part, int blocks,
                              hipStream_t st);

// Dense paths: the sum of the product's partials fused with lines 7-12 of Alg. 2 (see finalize_cg_kernel).
struct FinCgArgs {
    const CgSlot *prev;      // state before product k-1 (k >= 1), completed by that product's finalize
    CgSlot *cur;             // state before product k, written by block 0 (k == 0 with n_gg == 0: the initialisation's, read)
    int32_t first;           // k == 0
    const double *gg_part;   // k == 0: n_gg partials of g.g; the initial state (line 1 of Alg. 2) is formed from them here
    int n_gg;                //         0: slot *cur already holds the initial state
    double theta;
    void *pv, *r, *s, *hs, *pbest;   // CG vectors on the leading dimension FinArgs::ldm (FinArgs::M is not used)
    const double *zu_part;   // per-wave partials of sum_i z_i . u_i left by the product's launch (operand r_k)
    int n_zu;
    const double *rr_in, *rhs_in;    // partials of r_k.r_k and r_k.(H s_{k-1}) from the previous finalize (k >= 1)
    int n_in;
    double *rr_out, *rhs_out;        // out: one partial per block of r_{k+1}.r_{k+1} and r_{k+1}.(H s_k)
    double *trace;           // nullable: 3 doubles per product (alpha, ||r_new||, s^T H s)
    int32_t k;
};
hipError_t launch_finalize_cg(int dtype, const FinArgs &a, const FinCgArgs &g, int blocks, hipStream_t st);
// small blocks: lines 1-5 and the initial state in one launch (one block)
hipError_t launch_cg_init_small(int dtype, const CgVecs &v, CgSlot *slot0, hipStream_t st);
// inside ssn_solve: the tail, the slope <p_best, G>, the trial point W + p_best and the publication of F(x_k) (*f_dev),
// the slope and the final state to host-visible memory; one launch with blocks == 1, else two (slope_part: blocks
// partials)
hipError_t launch_cg_tail_solve(int dtype, const CgVecs &v, const CgSlot *prev, CgSlot *fin, const double *rr_in, int n_in,
                                double theta, double *trace, int k, const void *W, void *trial, const double *f_dev,
                                double *slope_dev, double *host_out, double *slope_part, int blocks, hipStream_t st);
// after the last product: the test of lines 10-11 for r_T, the pending p_best copy, the final state
hipError_t launch_cg_tail(int dtype, const CgVecs &v, const CgSlot *prev, CgSlot *fin, const double *rr_in, int n_in,
                          double theta, double *trace, int k, int blocks, hipStream_t st);

}  // namespace ssn
