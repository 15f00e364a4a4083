// extern "C" entry points of libssn_hip.so (declared in include/ssn.h): argument checking, workspace
// ownership, kernel sequencing, and the host-side control flow of Alg. 1 and Alg. 3.  Every arithmetic
// step runs in the kernels of dense_mfma.hip / csr.hip / csc.hip / vecops.hip / preprocess.hip.
#include "ssn_internal.h"
#include "ssn_bench.h"

#include <chrono>
#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace ssn;

struct ssn_ctx {
    ssn_desc d{};
    int K = 0, KP = 0;
    size_t es = 0;
    hipStream_t st = nullptr;
    int num_cus = 256;
    std::string err;

    // per-row buffers (row stride KP): U of the current product, P of the prepared sample
    void *Ubuf = nullptr;
    int64_t U_rows = 0;
    void *Pbuf = nullptr;
    int64_t P_rows = 0;
    // per-chunk partial sums of X^T U (dense path)
    void *part = nullptr;
    int64_t part_elems = 0;
    int max_chunks = 0;
    bool fused = false;           // dense: the one-pass kernel serves this shape
    bool binary = false;          // dense, K = 1: the matrix-vector kernels of dense_binary.hip serve every mode
    // sampled product on few row blocks of a wide matrix (two-kernel path): the last ROW_APPLY launch left partial
    // margins of z_slices feature slices in Ubuf instead of U, and the transposed product that follows forms U itself
    bool z_active = false;
    int z_slices = 0;
    // CSR: column-sorted views for the transposed products (whole matrix: built at the first gradient;
    // sample: rebuilt by every ssn_hess_prepare)
    CscView csc_full, csc_samp, csc_grad;      // csc_grad: the sample of the last sub-sampled gradient
    // ssn_solve builds the view of the NEXT iteration's sample (it depends on the sample only, not on the
    // iterate) on a stream of its own while the current iteration's line search runs
    CscView csc_next;
    hipStream_t st_aux = nullptr;
    hipEvent_t ev_aux = nullptr;
    const int32_t *next_S = nullptr;
    int64_t next_nS = 0;
    bool next_ready = false;
    bool csc_full_built = false;
    int32_t csr_max_len = 0;      // longest row of the CSR matrix (read when the whole matrix's view is built)
    // CSR with one weight column: what the lane-per-entry kernels of the full passes need (csr1_flat_kernel) -- the row
    // of every 64th stored entry, the rows' margins, the windows' leading partial sums
    int32_t *csr1_rwin = nullptr;
    void *csr1_zrow = nullptr, *csr1_zhead = nullptr;
    // reduction scratch
    double *loss_part = nullptr;
    int32_t *hit_part = nullptr;
    int wave_parts = 0;
    double *red_a = nullptr, *red_b = nullptr, *red_c = nullptr;
    double *red_sq = nullptr;                  // partials of ||M||^2 left by the kernel that made the block sq_for
    const void *sq_for = nullptr;
    int n_sq = 0;
    double *scal_dev = nullptr;
    int32_t *int_dev = nullptr;
    double *host_pin = nullptr;   // pinned staging for scalar results
    double *f_host = nullptr;     // host-visible word kernels write objective values to (inside host_pin's allocation)
    double *f_host_dev = nullptr; // its device address
    unsigned long long *f_ticket = nullptr, *f_ticket_dev = nullptr;   // ticket word next to f_host: the kernel posts the
                                  // value, then the ticket of its enqueue; the host spins on it instead of synchronising
    unsigned long long f_seq = 0; // ticket of the last enqueue
    double *pub_host = nullptr;   // host-visible block ssn_solve's per-iteration scalars and CG state are written to
    double *pub_dev = nullptr;    // its device address
    // prepared Hessian sample
    const int32_t *S = nullptr;
    int64_t nS = 0;
    bool prepared = false;
    // CG / line-search vectors (p x ldw each)
    void *cg_p = nullptr, *cg_r = nullptr, *cg_s = nullptr, *trial = nullptr;
    void *grad = nullptr, *dir = nullptr;      // ssn_solve's gradient and direction
    void *cg_hs = nullptr;                     // dense paths: H s, kept by recurrence (see finalize_cg_kernel)
    double *cg_parts = nullptr;                // dense paths: 2 x 2 x RED_MAX_PARTS partials of r.r and r.(H s), double-buffered
    void *cg_pb = nullptr;                     // CSR: best iterate on the sample's columns (cg_pb_cap elements)
    int64_t cg_pb_cap = 0;
    void *grad_next = nullptr;                 // gradient at the first line-search trial (look-ahead of ssn_solve)
    CgSlot *slots = nullptr;
    int slots_cap = 0;
    void *tail_row = nullptr;                  // dense one-pass path: zero-padded copy of row n-1 (tail_len elements)
    int tail_len = 0;
    int cg_gg_parts = 0;                       // dense CG: partials of g.g in red_a the first finalize forms slot 0 from (0: slot 0 is set)
    double *trace_dev = nullptr;
    // line search on cached margins: Z = [X W | X P] (n rows of 2K values) and the partials of W.W, W.P, P.P
    void *Zbuf = nullptr;
    double *ls_dots = nullptr;
};

namespace {

#define SSN_HIP(ctx, call)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e_);                        \
            return (e_ == hipErrorOutOfMemory) ? SSN_E_ALLOC : SSN_E_HIP;                          \
        }                                                                                          \
    } while (0)

#define SSN_TRY(expr)                                                                              \
    do {                                                                                           \
        int s_ = (expr);                                                                           \
        if (s_ != SSN_OK) return s_;                                                               \
    } while (0)

int fail(ssn_ctx *c, int code, const std::string &msg)
{
    if (c) c->err = msg;
    return code;
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

inline bool is_dense(const ssn_ctx *c) { return c->d.layout == SSN_DENSE_ROWMAJOR; }

double scale_full(const ssn_ctx *c) { return c->d.scale == SSN_SCALE_SUM ? 1.0 : 1.0 / (double)c->d.n; }
// data-term factor of a sum over nrows sampled rows (eqs. (2a), (2b))
double scale_rows(const ssn_ctx *c, int64_t nrows)
{
    return c->d.scale == SSN_SCALE_SUM ? (double)c->d.n / (double)nrows : 1.0 / (double)nrows;
}
double scale_sample(const ssn_ctx *c)
{
    return c->d.scale == SSN_SCALE_SUM ? (double)c->d.n / (double)c->nS : 1.0 / (double)c->nS;
}

int vec_bytes_alloc(ssn_ctx *c, void **ptr)
{
    SSN_HIP(c, hipMalloc(ptr, (size_t)c->d.p * (size_t)c->d.ldw * c->es));
    return SSN_OK;
}

// make sure a per-row buffer has at least `rows` rows
int ensure_rows(ssn_ctx *c, void **buf, int64_t *have, int64_t rows)
{
    if (*have >= rows) return SSN_OK;
    if (*buf) {
        SSN_HIP(c, hipStreamSynchronize(c->st));
        SSN_HIP(c, hipFree(*buf));
        *buf = nullptr;
        *have = 0;
    }
    SSN_HIP(c, hipMalloc(buf, (size_t)rows * (size_t)c->KP * c->es));
    *have = rows;
    return SSN_OK;
}

RowsArgs rows_base(const ssn_ctx *c)
{
    RowsArgs a{};
    a.X = c->d.X;
    a.ldx = c->d.ldx;
    a.rowptr = c->d.rowptr;
    a.colidx = c->d.colidx;
    a.vals = c->d.vals;
    a.n = c->d.n;
    a.p = c->d.p;
    a.K = c->K;
    a.labels = c->d.labels;
    a.KP = c->KP;
    a.ldm = c->d.ldw;
    a.loss_part = c->loss_part;
    a.hit_part = c->hit_part;
    a.tail_row = c->tail_row;
    a.tail_len = c->tail_len;
    return a;
}

XtuArgs xtu_base(const ssn_ctx *c)
{
    XtuArgs a{};
    a.X = c->d.X;
    a.ldx = c->d.ldx;
    a.rowptr = c->d.rowptr;
    a.colidx = c->d.colidx;
    a.vals = c->d.vals;
    a.n = c->d.n;
    a.p = c->d.p;
    a.K = c->K;
    a.KP = c->KP;
    a.part = c->part;
    return a;
}

// The one-pass kernel serves a launch when the shape allows it and it pays: always for the modes with a
// transposed product; for the margins-only modes with a multi-wave feature split, or on enough rows to
// give every single-wave workgroup a row block (on fewer rows of a narrow matrix the wave-per-row-block
// kernel is faster).
bool use_fused(const ssn_ctx *c, const RowsArgs &a)
{
    if (!c->fused || a.mode == ROW_MARGIN) return false;
    if (a.mode == ROW_GRAD || a.mode == ROW_APPLY) return true;
    if (dense_narrow_applies(c->d.dtype, a)) return true;        // long pass over a narrow matrix: the vector-unit kernel
    if (dense_fused_waves(c->d.dtype, a) > 1) return true;
    // narrow matrix, margins only: the one-pass kernel's single-wave workgroups win once every one of them has a
    // row block of its own to stream (workload 3, fp64 objective: 78 -> 62 us); on fewer rows the plain kernel does
    return a.nrows >= (int64_t)16 * 12 * c->num_cus;
}

// K = 1 on a dense matrix of at least 128 features: matrix-vector kernels instead of the 16-column matrix-core tiles
// (narrower matrices keep the tiles: a wave per row would idle most of its lanes).  SSN_BINARY_PATH=mfma turns it off
// (for measurements).
bool binary_path(const ssn_desc *d)
{
    const char *force = getenv("SSN_BINARY_PATH");
    return d->layout == SSN_DENSE_ROWMAJOR && d->C == 2 && d->p >= 128 && !(force && strcmp(force, "mfma") == 0);
}

hipError_t launch_xtu(const ssn_ctx *c, const XtuArgs &x)
{
    return c->binary ? launch_binary_xtu(c->d.dtype, x, c->st) : launch_dense_xtu(c->d.dtype, x, c->st);
}

// A product on a sample with fewer row blocks than twice the compute units, on a wide matrix of the two-kernel path:
// the margins are computed per (row block, feature slice) so that every compute unit has work, and the transposed
// product forms U from the slices' partial margins (dense_zpart_kernel, dense_xtu_kernel<FROMZ>).  Returns the number
// of slices (0: the plain kernels serve) and the features per slice.
int zpart_plan(const ssn_ctx *c, int64_t nrows, int64_t *fper)
{
    static const bool off = [] { const char *e = getenv("SSN_SAMPLED_SLICES"); return e && e[0] == '0'; }();
    if (off || !is_dense(c) || c->fused || c->binary || c->K > 16 || c->d.p < 512) return 0;
    if ((uintptr_t)c->d.X % 16 != 0 || (c->d.ldx * (int64_t)c->es) % 16 != 0) return 0;
    const int64_t nblk = (nrows + 15) / 16;
    if (nblk > (int64_t)c->num_cus * 2) return 0;
    int64_t slices = ((int64_t)c->num_cus * 2) / nblk;
    if (slices > c->d.p / 256) slices = c->d.p / 256;            // at least 256 features per slice
    if (slices > 4) slices = 4;                                  // what the transposed-product kernel adds up
    if (slices < 2) return 0;
    const int64_t per = round_up((c->d.p + slices - 1) / slices, 64);
    slices = (c->d.p + per - 1) / per;
    if (slices < 2 || slices * round_up(nrows, 16) > c->U_rows) return 0;      // the partial margins live in the U buffer
    *fper = per;
    return (int)slices;
}

// the transposed product after a ROW_APPLY launch: U from the buffer, or formed from the slices' partial margins
void xtu_after_apply(const ssn_ctx *c, XtuArgs *x)
{
    x->U = c->Ubuf;
    if (!c->z_active) return;
    x->Zpart = c->Ubuf;
    x->nslices = c->z_slices;
    x->zrows = round_up(x->nrows, 16);
    x->Pin = c->Pbuf;
    x->zu_part = c->loss_part;
}

int launch_rows(ssn_ctx *c, const RowsArgs &a, int *nparts)
{
    if (a.mode == ROW_APPLY) {
        int64_t fper = 0;
        const int slices = zpart_plan(c, a.nrows, &fper);
        c->z_active = slices > 0;
        c->z_slices = slices;
        if (slices > 0) {
            SSN_HIP(c, launch_dense_zpart(c->d.dtype, a, c->Ubuf, slices, fper, c->st));
            if (nparts) *nparts = 0;         // the sums of z_i . u_i come from the transposed product: one per row chunk
            return SSN_OK;
        }
    }
    if (c->binary) {
        const int blocks = binary_rows_blocks(a.nrows, c->num_cus);
        if (blocks * ROWS_WAVES_PER_BLOCK > c->wave_parts) return fail(c, SSN_E_INVALID_ARG, "internal: wave partial overflow");
        SSN_HIP(c, launch_binary_rows(c->d.dtype, a, blocks, c->st));
        if (nparts) *nparts = blocks * ROWS_WAVES_PER_BLOCK;
        return SSN_OK;
    }
    if (use_fused(c, a)) {
        const int grid = dense_fused_grid(c->d.dtype, a, c->num_cus);
        if (grid * 4 > c->wave_parts || grid > c->max_chunks) return fail(c, SSN_E_INVALID_ARG, "internal: partial overflow");
        SSN_HIP(c, launch_dense_fused(c->d.dtype, a, grid, c->st));
        if (nparts) *nparts = grid * 4;          // loss / hit partials; the X^T U partials number `grid`
        return SSN_OK;
    }
    // dense: one wave per 16-row block; CSR: one wave per row
    int blocks = rows_grid_blocks(is_dense(c) ? a.nrows : a.nrows * 16, c->num_cus), split_waves = 0;
    // few row blocks of a wide matrix: a workgroup per row block (needs 16-byte aligned rows)
    if (is_dense(c) && (uintptr_t)c->d.X % 16 == 0 && (c->d.ldx * (int64_t)c->es) % 16 == 0)
        dense_rows_plan(c->d.dtype, a.nrows, c->d.p, a.mode == ROW_MARGIN ? 2 * c->K : c->K, c->num_cus, &blocks, &split_waves);
    if (!is_dense(c)) {
        // rows differ in length, so more waves than fit on the chip at once let the hardware fill in behind the short
        // ones (sparse workload: objective 248 -> 237 us in fp64, 137 -> 124 us in fp32 against eight per compute unit)
        const int64_t cap = (int64_t)c->num_cus * 16, want = (a.nrows + ROWS_WAVES_PER_BLOCK - 1) / ROWS_WAVES_PER_BLOCK;
        blocks = (int)(want < cap ? want : cap);
        if (blocks < 1) blocks = 1;
        // one weight column, every row of the matrix: a lane per stored entry (csr1_flat_kernel)
        if (c->K == 1 && c->csr1_rwin && !a.S && a.nrows == c->d.n && a.rowptr == c->d.rowptr && a.colidx == c->d.colidx &&
            a.vals == c->d.vals && (a.mode == ROW_OBJ || a.mode == ROW_GRAD || a.mode == ROW_PRED)) {
            RowsArgs b = a;
            b.rwin = c->csr1_rwin;
            b.zrow = c->csr1_zrow;
            b.zhead = c->csr1_zhead;
            b.nnz = c->d.nnz;
            // the per-row kernel takes a row per lane: a workgroup per 256 rows (and that many fewer partial sums)
            const int64_t rb = (a.nrows + 64 * ROWS_WAVES_PER_BLOCK - 1) / (64 * ROWS_WAVES_PER_BLOCK);
            if (rb < blocks) blocks = (int)(rb < 1 ? 1 : rb);
            if (blocks * ROWS_WAVES_PER_BLOCK > c->wave_parts) return fail(c, SSN_E_INVALID_ARG, "internal: wave partial overflow");
            SSN_HIP(c, launch_csr_rows(c->d.dtype, b, blocks, c->st));
            if (nparts) *nparts = blocks * ROWS_WAVES_PER_BLOCK;
            return SSN_OK;
        }
        // Few, long rows (the sampled rows of the products, on a matrix of hundreds of entries per row): a workgroup
        // per row, whose four waves share the row's entries -- a wave per row would leave most SIMDs without a wave
        // and give each wave a long chain of rounds.
        if (c->K > 1 && (a.mode == ROW_APPLY || a.mode == ROW_PREP) && a.nrows <= (int64_t)c->num_cus * 8 &&
            c->d.n > 0 && c->d.nnz / c->d.n >= 128) {
            RowsArgs b = a;
            b.csr_split = 1;
            blocks = (int)(a.nrows < cap ? a.nrows : cap);
            if (blocks < 1) blocks = 1;
            if (blocks * ROWS_WAVES_PER_BLOCK > c->wave_parts) return fail(c, SSN_E_INVALID_ARG, "internal: wave partial overflow");
            SSN_HIP(c, launch_csr_rows(c->d.dtype, b, blocks, c->st));
            if (nparts) *nparts = blocks * ROWS_WAVES_PER_BLOCK;
            return SSN_OK;
        }
    }
    if (blocks * ROWS_WAVES_PER_BLOCK > c->wave_parts) return fail(c, SSN_E_INVALID_ARG, "internal: wave partial overflow");
    if (is_dense(c)) SSN_HIP(c, launch_dense_rows(c->d.dtype, a, blocks, split_waves, c->st));
    else SSN_HIP(c, launch_csr_rows(c->d.dtype, a, blocks, c->st));
    if (nparts) *nparts = blocks * ROWS_WAVES_PER_BLOCK;
    return SSN_OK;
}

// Waves of the transposed-product kernel to aim at per compute unit.  A narrow matrix has a single
// 64-feature tile, so all the parallelism comes from row chunks and each wave is a short chain of loads:
// more, shorter chunks keep more loads in flight.  Wider matrices: three waves per SIMD (50000 x 3072, all rows:
// 216 us in fp64 and 108 us in fp32, against 247 / 122 us with two and 224 / 112 us with five).
int xtu_waves_per_cu(int64_t p) { return p <= 128 ? 32 : 12; }

// choose the row chunking of the dense transposed product
void choose_chunks(const ssn_ctx *c, int64_t nrows, int64_t *rpc, int *nch)
{
    if (c->binary) {
        // a block of the matrix-vector kernel covers 256 sixteen-byte vectors of features; aim at 8 blocks per
        // compute unit, chunks of at least 8 rows
        const int64_t tiles = (c->d.p * (int64_t)c->es + 4095) / 4096;
        int64_t n = ((int64_t)c->num_cus * 8 + tiles - 1) / tiles;
        if (n > (nrows + 7) / 8) n = (nrows + 7) / 8;
        if (n > c->max_chunks) n = c->max_chunks;
        if (n < 1) n = 1;
        const int64_t r = (nrows + n - 1) / n;
        *rpc = r;
        *nch = (int)((nrows + r - 1) / r);
        return;
    }
    const int64_t nft = (c->d.p + 63) / 64;
    const int64_t target = (int64_t)c->num_cus * xtu_waves_per_cu(c->d.p);
    int64_t n = (target + nft - 1) / nft;
    const int64_t maxn = (nrows + 15) / 16;
    if (n > maxn) n = maxn;
    if (n > c->max_chunks) n = c->max_chunks;
    if (n < 1) n = 1;
    int64_t r = round_up((nrows + n - 1) / n, 16);
    *rpc = r;
    *nch = (int)((nrows + r - 1) / r);
}

// out = scale * sum of the `nchunks` partials in c->part + lambda * M ; optionally partials of <out, M>
int finalize_dense(ssn_ctx *c, int nchunks, double scale, const void *M, void *out, bool want_dot, int *ndot,
                   const int32_t *skip)
{
    FinArgs f{};
    f.part = c->part;
    f.nchunks = nchunks;
    f.p = c->d.p;
    f.K = c->K;
    f.scale = scale;
    f.lambda = c->d.lambda;
    f.M = M;
    f.ldm = c->d.ldw;
    f.out = out;
    f.ldo = c->d.ldw;
    f.dot_part = want_dot ? c->red_b : nullptr;
    f.skip = skip;
    const int fb = finalize_blocks(c->d.p, c->K);
    SSN_HIP(c, launch_finalize(c->d.dtype, f, fb, c->st));
    if (ndot) *ndot = fb;
    return SSN_OK;
}

// CSR: the column-sorted view of the rows a transposed product runs over (S == nullptr: the whole matrix,
// built on first use; otherwise the prepared sample's)
int csc_view_for(ssn_ctx *c, const int32_t *S, const CscView **view)
{
    if (S) {
        *view = &c->csc_samp;
        return SSN_OK;
    }
    if (!c->csc_full_built) {
        SSN_HIP(c, csc_build(&c->csc_full, c->d.dtype, c->d.rowptr, c->d.colidx, c->d.vals, nullptr, c->d.n, c->d.p, c->K,
                             c->st));
        // the sort's permutation (sorted place -> place in the CSR arrays) stays: samples' views are filtered out
        // of this one and need it
        c->csc_full.csr_pos = c->csc_full.idx_out;
        c->csc_full.idx_out = nullptr;
        csc_free_scratch(&c->csc_full);
        SSN_HIP(c, csr_max_row_len(c->d.rowptr, c->d.n, c->int_dev, &c->csr_max_len, c->st));
        if (c->K == 1) SSN_HIP(c, csc_window_index(&c->csc_full, c->st));
        c->csc_full_built = true;
    }
    *view = &c->csc_full;
    return SSN_OK;
}

// CSR: the column-sorted view of a sample.  Filtered out of the whole matrix's view (no sort; built first if it
// is not there yet) unless the row lengths are too uneven for that path's buffer bound or SSN_CSR_VIEW=sort asks
// for the sorting construction.
static int build_sample_view(ssn_ctx *c, CscView *v, const int32_t *S, int64_t nS, hipStream_t st, bool support)
{
    const char *env = getenv("SSN_CSR_VIEW");       // read at every call: tests switch between the constructions
    const bool force_sort = env && env[0] == 's';
    if (!force_sort) {
        const CscView *full = nullptr;
        SSN_TRY(csc_view_for(c, nullptr, &full));
        const hipError_t e = csc_build_filtered(v, *full, c->d.dtype, c->d.rowptr, c->d.colidx, c->d.vals, S, nS, c->d.n,
                                                c->csr_max_len, c->K, st, support);
        if (e == hipSuccess) {
            if (c->K == 1) SSN_HIP(c, csc_window_index(v, st));
            return SSN_OK;
        }
        if (e != hipErrorNotSupported) SSN_HIP(c, e);
    }
    SSN_HIP(c, csc_build(v, c->d.dtype, c->d.rowptr, c->d.colidx, c->d.vals, S, nS, c->d.p, c->K, st, support));
    if (c->K == 1) SSN_HIP(c, csc_window_index(v, st));
    return SSN_OK;
}

// out = scale * X_rows^T U + lambda * M ; optionally partials of <out, M> into red_b (count in *ndot)
// after_apply: the rows kernel before it was a ROW_APPLY launch (see xtu_after_apply)
int transposed_product(ssn_ctx *c, const int32_t *S, int64_t nrows, double scale, const void *M, void *out,
                       bool want_dot, int *ndot, const int32_t *skip, const CscView *view_in = nullptr,
                       bool after_apply = false)
{
    XtuArgs x = xtu_base(c);
    x.S = S;
    x.nrows = nrows;
    x.U = c->Ubuf;
    x.skip = skip;
    if (is_dense(c)) {
        choose_chunks(c, nrows, &x.rows_per_chunk, &x.nchunks);
        if (after_apply) xtu_after_apply(c, &x);
        SSN_HIP(c, launch_xtu(c, x));
        SSN_TRY(finalize_dense(c, x.nchunks, scale, M, out, want_dot, ndot, skip));
    } else {
        const CscView *view = view_in;
        if (!view) SSN_TRY(csc_view_for(c, S, &view));
        SSN_HIP(c, launch_scale_copy(c->d.dtype, c->d.p, c->K, c->d.lambda, M, c->d.ldw, out, c->d.ldw, skip, c->st));
        SSN_HIP(c, launch_csc_apply(c->d.dtype, *view, c->K, c->KP, c->Ubuf, scale, out, c->d.ldw, nullptr, skip, c->st));
        if (want_dot) {
            const int vb = vec_blocks(c->d.p * (int64_t)c->K);
            SSN_HIP(c, launch_dot_part(c->d.dtype, c->d.p, c->K, out, c->d.ldw, M, c->d.ldw, c->red_b, vb, skip, c->st));
            if (ndot) *ndot = vb;
        }
    }
    return SSN_OK;
}

int read_scalar(ssn_ctx *c, const double *dev, double *host_out)
{
    SSN_HIP(c, hipMemcpyAsync(c->host_pin, dev, sizeof(double), hipMemcpyDeviceToHost, c->st));
    SSN_HIP(c, hipStreamSynchronize(c->st));
    *host_out = c->host_pin[0];
    return SSN_OK;
}

int read_int(ssn_ctx *c, const int32_t *dev, int32_t *host_out)
{
    SSN_HIP(c, hipMemcpyAsync(c->host_pin, dev, sizeof(int32_t), hipMemcpyDeviceToHost, c->st));
    SSN_HIP(c, hipStreamSynchronize(c->st));
    *host_out = *(const int32_t *)c->host_pin;
    return SSN_OK;
}

// enqueue f(W) into scal_dev[slot]; loss partials must already be in loss_part[0..nparts)
// f(W) into scal_dev[slot] from the loss partials the rows kernel left.  *mirrored (nullable) tells whether the
// value also lands in the host-visible word c->f_host (small blocks: one launch does everything).
// dst (nullable): the caller's device word receives the value instead of scal_dev[slot], and nothing is posted to the host
int enqueue_objective_value(ssn_ctx *c, const void *W, int nparts, int slot, double scale = -1.0, bool *mirrored = nullptr,
                            double *dst = nullptr)
{
    if (scale < 0.0) scale = scale_full(c);
    if (mirrored) *mirrored = false;
    // the host-visible copy and its ticket go with slot 0 only (the value a caller is about to wait for)
    const bool post = slot == 0 && !dst;
    if (!dst) dst = c->scal_dev + slot;
    double *oh = post ? c->f_host_dev : nullptr;
    unsigned long long *th = post ? c->f_ticket_dev : nullptr;
    const unsigned long long ticket = post ? ++c->f_seq : 0;
    if (mirrored) *mirrored = post;
    if (c->d.p * (int64_t)c->K <= OBJ_VALUE_ELEMS) {
        SSN_HIP(c, launch_objective_value(c->d.dtype, c->loss_part, nparts, scale, W, c->d.p, c->K, c->d.ldw,
                                          0.5 * c->d.lambda, dst, oh, th, ticket, c->st));
        return SSN_OK;
    }
    if (c->sq_for == W && c->n_sq > 0) {         // the kernel that wrote W left the partials of ||W||^2
        c->sq_for = nullptr;
        SSN_HIP(c, launch_combine(c->loss_part, nparts, scale, c->red_sq, c->n_sq, 0.5 * c->d.lambda, dst, c->st, oh, th,
                                  ticket));
        return SSN_OK;
    }
    const int vb = vec_blocks(c->d.p * (int64_t)c->K);
    SSN_HIP(c, launch_dot_part(c->d.dtype, c->d.p, c->K, W, c->d.ldw, W, c->d.ldw, c->red_a, vb, nullptr, c->st));
    SSN_HIP(c, launch_combine(c->loss_part, nparts, scale, c->red_a, vb, 0.5 * c->d.lambda, dst, c->st, oh, th, ticket));
    return SSN_OK;
}

double now_ms();

// wait for f(W) enqueued by enqueue_objective_value into scal_dev[0]
int read_objective(ssn_ctx *c, bool mirrored, double *f)
{
    if (mirrored) {
        // Spin on the ticket the value kernel posts behind the value.  Everything enqueued before that kernel
        // has completed by then (one stream), and the host is back a microsecond or two after the store instead
        // of a stream synchronisation's wake-up later.  A ticket that does not come (a failed launch, a fault)
        // ends in the synchronisation, which reports it.
        const unsigned long long want = c->f_seq;
        const double t_give_up = now_ms() + 2000.0;
        bool seen = false;
        for (unsigned spin = 0;; ++spin) {
            if (__atomic_load_n(c->f_ticket, __ATOMIC_ACQUIRE) == want) { seen = true; break; }
            if ((spin & 0x3ff) == 0x3ff && now_ms() > t_give_up) break;
        }
        if (!seen) SSN_HIP(c, hipStreamSynchronize(c->st));
        *f = *(volatile double *)c->f_host;
    } else {
        SSN_TRY(read_scalar(c, c->scal_dev, f));
    }
    if (!std::isfinite(*f)) return fail(c, SSN_E_NONFINITE, "objective is not finite");
    return SSN_OK;
}

// enqueue F(W) over all rows into scal_dev[0] (and the host-visible word when *mirrored comes back true)
int objective_enqueue(ssn_ctx *c, const void *W, bool *mirrored)
{
    RowsArgs a = rows_base(c);
    a.nrows = c->d.n;
    a.M = W;
    a.mode = ROW_OBJ;
    int nparts = 0;
    SSN_TRY(launch_rows(c, a, &nparts));
    return enqueue_objective_value(c, W, nparts, 0, -1.0, mirrored);
}

int objective_impl(ssn_ctx *c, const void *W, double *f)
{
    bool mirrored = false;
    SSN_TRY(objective_enqueue(c, W, &mirrored));
    return read_objective(c, mirrored, f);
}

// defer_f: leave f(W) in scal_dev[0] without reading it back (the caller synchronises later).
// S (nullable): the sub-sampled gradient of eq. (2a) on the nS rows S, with its sample scaling.
// f_dev (nullable): f(W) goes to that device word instead (nothing is read back, nothing posted to the host).
int gradient_impl(ssn_ctx *c, const void *W, void *G, double *f, bool defer_f = false, const int32_t *S = nullptr,
                  int64_t nS = 0, bool *mirrored_out = nullptr, double *f_dev = nullptr)
{
    const int64_t nrows = S ? nS : c->d.n;
    const double scale = S ? scale_rows(c, nS) : scale_full(c);
    if (!c->fused) SSN_TRY(ensure_rows(c, &c->Ubuf, &c->U_rows, round_up(nrows, 16)));
    RowsArgs a = rows_base(c);
    a.S = S;
    a.nrows = nrows;
    a.M = W;
    a.mode = ROW_GRAD;
    a.UP = c->Ubuf;
    int nparts = 0;
    a.part = c->part;
    SSN_TRY(launch_rows(c, a, &nparts));
    if (c->fused) {
        SSN_TRY(finalize_dense(c, nparts / 4, scale, W, G, false, nullptr, nullptr));
    } else {
        const CscView *view = nullptr;
        if (!is_dense(c) && S) {             // a view of its own: the prepared Hessian sample keeps csc_samp
            SSN_TRY(build_sample_view(c, &c->csc_grad, S, nS, c->st, false));
            view = &c->csc_grad;
        }
        SSN_TRY(transposed_product(c, S, nrows, scale, W, G, false, nullptr, nullptr, view));
    }
    bool mirrored = false;
    if (f_dev) return enqueue_objective_value(c, W, nparts, 0, scale, nullptr, f_dev);
    if (f || defer_f) SSN_TRY(enqueue_objective_value(c, W, nparts, 0, scale, &mirrored));
    if (f && !defer_f) SSN_TRY(read_objective(c, mirrored, f));
    if (mirrored_out) *mirrored_out = mirrored;
    return SSN_OK;
}

// HV = H_S V.  want_dot: partials of <HV, V> into red_b (count in *ndot).
int hess_apply_impl(ssn_ctx *c, const void *V, void *HV, bool want_dot, int *ndot, const int32_t *skip)
{
    RowsArgs a = rows_base(c);
    a.S = c->S;
    a.nrows = c->nS;
    a.M = V;
    a.mode = ROW_APPLY;
    a.Pin = c->Pbuf;
    a.UP = c->Ubuf;
    a.skip = skip;
    a.part = c->part;
    int nparts = 0;
    SSN_TRY(launch_rows(c, a, &nparts));
    if (c->fused) return finalize_dense(c, nparts / 4, scale_sample(c), V, HV, want_dot, ndot, skip);
    return transposed_product(c, c->S, c->nS, scale_sample(c), V, HV, want_dot, ndot, skip, nullptr, true);
}

// Product k of the CG loop with the vector updates of Alg. 2 behind it.  H s is never formed by a product of
// its own.  Dense paths: the product is applied to r_k and finalize_cg_kernel does lines 7-12 (two launches
// per iteration on the one-pass path); the state before product k is completed in slots[k] by that kernel.
// CSR path: alpha, r -= alpha H s here, p and s in step 2 (*p_pending); the curvature
// s^T H s = scale * sum_i z_i . u_i + lambda * s.s comes from the per-wave partials the rows kernel leaves in
// loss_part and the partials of s.s in red_c (n_ss of them); on return red_a holds *n_rr partials of the new r.r.
int cg_product_step(ssn_ctx *c, const CgVecs &v, CgSlot *slots, int k, double theta, int n_ss, double *trace, int *n_rr,
                    bool *p_pending)
{
    CgSlot *cur = slots + k;
    // dense paths: the theta test for r_k is made by product k's own finalize, so the flag the product's
    // launches look at is the one before it
    const CgSlot *flag_slot = (is_dense(c) && k > 0) ? slots + (k - 1) : cur;
    const int32_t *skip = (const int32_t *)((const char *)flag_slot + offsetof(CgSlot, done));
    const bool form_state = is_dense(c) && k == 0 && c->cg_gg_parts > 0;     // slot 0 is written behind product 0
    if (form_state) skip = nullptr;
    double *trace_k = trace + 3 * k;
    RowsArgs a = rows_base(c);
    a.S = c->S;
    a.nrows = c->nS;
    a.M = is_dense(c) ? v.r : v.s;
    a.mode = ROW_APPLY;
    a.Pin = c->Pbuf;
    a.UP = c->Ubuf;
    a.skip = skip;
    a.part = c->part;
    if (!is_dense(c)) {
        // the sample's rows as a CSR matrix over the columns they touch (the CG vectors live there)
        const CscView &sv = c->csc_samp;
        a.S = nullptr;
        a.rowptr = sv.off;
        a.colidx = sv.ccol;
        a.vals = sv.val_in;
        a.p = v.p;
        a.ldm = v.ld;
    }
    int nparts = 0;
    SSN_TRY(launch_rows(c, a, &nparts));
    *p_pending = false;
    if (is_dense(c)) {
        int nchunks = nparts / 4;
        if (!c->fused) {
            XtuArgs x = xtu_base(c);
            x.S = c->S;
            x.nrows = c->nS;
            x.skip = skip;
            choose_chunks(c, c->nS, &x.rows_per_chunk, &x.nchunks);
            xtu_after_apply(c, &x);
            SSN_HIP(c, launch_xtu(c, x));
            nchunks = x.nchunks;
            if (c->z_active) nparts = nchunks;       // one sum of z_i . u_i per row chunk
        }
        FinArgs f{};
        f.part = c->part;
        f.nchunks = nchunks;
        f.p = c->d.p;
        f.K = c->K;
        f.scale = scale_sample(c);
        f.lambda = c->d.lambda;
        f.ldm = c->d.ldw;
        const int fb = finalize_blocks(c->d.p, c->K);
        double *in = c->cg_parts + (size_t)((k + 1) & 1) * 2 * RED_MAX_PARTS;
        double *out = c->cg_parts + (size_t)(k & 1) * 2 * RED_MAX_PARTS;
        FinCgArgs g{};
        g.prev = k > 0 ? slots + (k - 1) : nullptr;
        g.cur = cur;
        g.first = k == 0;
        g.gg_part = form_state ? c->red_a : nullptr;
        g.n_gg = form_state ? c->cg_gg_parts : 0;
        g.theta = theta;
        g.pv = v.pv;
        g.r = v.r;
        g.s = v.s;
        g.hs = c->cg_hs;
        g.pbest = v.pbest;
        g.zu_part = c->loss_part;
        g.n_zu = nparts;
        g.rr_in = in;
        g.rhs_in = in + RED_MAX_PARTS;
        g.n_in = fb;
        g.rr_out = out;
        g.rhs_out = out + RED_MAX_PARTS;
        g.trace = trace;
        g.k = k;
        SSN_HIP(c, launch_finalize_cg(c->d.dtype, f, g, fb, c->st));
        *n_rr = fb;
        return SSN_OK;
    }
    // CSR: alpha first, then the few entries of r the sample's columns touch, then one dense pass over r and s
    SSN_HIP(c, launch_cg_alpha(cur, c->loss_part, nparts, c->red_c, n_ss, scale_sample(c), c->d.lambda, trace_k, c->st));
    SSN_HIP(c, launch_csc_apply(c->d.dtype, c->csc_samp, c->K, c->KP, c->Ubuf, scale_sample(c), v.r, v.ld, cur, skip,
                                c->st, true));
    const int vb = vec_blocks(v.p * (int64_t)c->K);
    SSN_HIP(c, launch_cg_r_update(c->d.dtype, v, cur, c->d.lambda, c->red_a, vb, c->st));
    *n_rr = vb;
    *p_pending = true;
    return SSN_OK;
}

double now_ms()
{
    using namespace std::chrono;
    return duration<double, std::milli>(steady_clock::now().time_since_epoch()).count();
}

}  // namespace

extern "C" {

const char *ssn_strerror(int status)
{
    switch (status) {
    case SSN_OK: return "ok";
    case SSN_E_INVALID_ARG: return "invalid argument";
    case SSN_E_BAD_LABEL: return "label outside [0,C)";
    case SSN_E_BAD_INDEX: return "index out of range";
    case SSN_E_NOT_PREPARED: return "Hessian sample not prepared";
    case SSN_E_ALLOC: return "device allocation failed";
    case SSN_E_HIP: return "HIP runtime error";
    case SSN_E_NONFINITE: return "non-finite objective";
    case SSN_E_UNSUPPORTED: return "unsupported shape";
    case SSN_E_TOO_LARGE: return "problem exceeds the fixed workspace of ssn_hessvec_static";
    default: return "unknown status";
    }
}

const char *ssn_last_error(const ssn_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int ssn_normalize_columns(int32_t layout, int32_t dtype, int64_t n, int64_t p, void *X, int64_t ldx, const int32_t *rowptr,
                          const int32_t *colidx, void *vals, int64_t nnz, double *colnorm, void *stream)
{
    if (n < 1 || p < 1 || !colnorm || (dtype != SSN_F32 && dtype != SSN_F64)) return SSN_E_INVALID_ARG;
    if (n >= (int64_t)1 << 31 || p >= (int64_t)1 << 31) return SSN_E_UNSUPPORTED;
    if (layout == SSN_DENSE_ROWMAJOR) {
        if (!X || ldx < p) return SSN_E_INVALID_ARG;
    } else if (layout == SSN_CSR) {
        if (!rowptr || nnz < 0 || (nnz > 0 && (!colidx || !vals))) return SSN_E_INVALID_ARG;
        if (nnz >= (int64_t)1 << 31) return SSN_E_UNSUPPORTED;
    } else {
        return SSN_E_INVALID_ARG;
    }
    const hipError_t e = normalize_columns(layout, dtype, n, p, X, ldx, rowptr, colidx, vals, nnz, colnorm, (hipStream_t)stream);
    if (e == hipSuccess) return SSN_OK;
    return e == hipErrorOutOfMemory ? SSN_E_ALLOC : SSN_E_HIP;
}

int ssn_destroy(ssn_ctx *c)
{
    if (!c) return SSN_E_INVALID_ARG;
    (void)hipStreamSynchronize(c->st);
    if (c->st_aux) (void)hipStreamSynchronize(c->st_aux);      // a view of the next sample may still be in the making
    void *dev[] = {c->Zbuf, c->ls_dots, c->Ubuf, c->Pbuf, c->part, c->loss_part, c->hit_part, c->red_a, c->red_b, c->red_c, c->red_sq, c->scal_dev, c->int_dev,
                   c->cg_p, c->cg_r, c->cg_s, c->cg_hs, c->cg_parts, c->cg_pb, c->trial, c->grad, c->grad_next, c->dir, c->slots, c->trace_dev,
                   c->tail_row, c->csr1_rwin, c->csr1_zrow, c->csr1_zhead};
    for (void *p : dev)
        if (p) (void)hipFree(p);
    if (c->host_pin) (void)hipHostFree(c->host_pin);
    csc_free(&c->csc_full);
    csc_free(&c->csc_samp);
    csc_free(&c->csc_grad);
    csc_free(&c->csc_next);
    if (c->ev_aux) (void)hipEventDestroy(c->ev_aux);
    if (c->st_aux) (void)hipStreamDestroy(c->st_aux);
    delete c;
    return SSN_OK;
}

int ssn_create(ssn_ctx **out, const ssn_desc *d)
{
    if (!out || !d) return SSN_E_INVALID_ARG;
    *out = nullptr;
    if (d->n < 1 || d->p < 1 || d->C < 2 || !(d->lambda >= 0.0) || !d->labels) return SSN_E_INVALID_ARG;
    if (d->dtype != SSN_F32 && d->dtype != SSN_F64) return SSN_E_INVALID_ARG;
    if (d->scale != SSN_SCALE_MEAN && d->scale != SSN_SCALE_SUM) return SSN_E_INVALID_ARG;
    const int K = d->C - 1;
    if (d->ldw < K) return SSN_E_INVALID_ARG;
    if (d->n >= (int64_t)1 << 31 || d->p >= (int64_t)1 << 31) return SSN_E_UNSUPPORTED;
    if (d->layout == SSN_DENSE_ROWMAJOR) {
        if (!d->X || d->ldx < d->p) return SSN_E_INVALID_ARG;
        if (K > 32) return SSN_E_UNSUPPORTED;
    } else if (d->layout == SSN_CSR) {
        if (!d->rowptr || d->nnz < 0 || (d->nnz > 0 && (!d->colidx || !d->vals))) return SSN_E_INVALID_ARG;
        if (d->nnz >= (int64_t)1 << 31) return SSN_E_UNSUPPORTED;
        if (K > 64) return SSN_E_UNSUPPORTED;
    } else {
        return SSN_E_INVALID_ARG;
    }

    ssn_ctx *c = new (std::nothrow) ssn_ctx();
    if (!c) return SSN_E_ALLOC;
    c->d = *d;
    c->K = K;
    c->es = d->dtype == SSN_F32 ? 4 : 8;
    c->KP = d->layout == SSN_DENSE_ROWMAJOR ? (K + 15) / 16 * 16 : K;
    c->st = (hipStream_t)d->stream;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        c->num_cus = prop.multiProcessorCount;

    auto bail = [&](int code) {
        ssn_destroy(c);
        return code;
    };
#define CREATE_HIP(call)                                                                           \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return bail(e_ == hipErrorOutOfMemory ? SSN_E_ALLOC : SSN_E_HIP);   \
    } while (0)

    c->wave_parts = c->num_cus * 16 * ROWS_WAVES_PER_BLOCK;
    CREATE_HIP(hipMalloc((void **)&c->loss_part, sizeof(double) * c->wave_parts));
    CREATE_HIP(hipMalloc((void **)&c->hit_part, sizeof(int32_t) * c->wave_parts));
    CREATE_HIP(hipMalloc((void **)&c->red_a, sizeof(double) * RED_MAX_PARTS));
    CREATE_HIP(hipMalloc((void **)&c->red_b, sizeof(double) * RED_MAX_PARTS));
    CREATE_HIP(hipMalloc((void **)&c->red_c, sizeof(double) * RED_MAX_PARTS));
    CREATE_HIP(hipMalloc((void **)&c->red_sq, sizeof(double) * RED_MAX_PARTS));
    CREATE_HIP(hipMalloc((void **)&c->scal_dev, sizeof(double) * 8));
    CREATE_HIP(hipMalloc((void **)&c->int_dev, sizeof(int32_t) * 8));
    CREATE_HIP(hipHostMalloc((void **)&c->host_pin, 4096));
    c->f_host = c->host_pin + 256;                                   // bytes 2048.. of the pinned page
    *c->f_host = 0.0;
    {
        // kernels post scalar results straight into this page: without a device mapping of it the context is
        // not created (there is no second, copy-based route to keep in step with the first)
        void *dp = nullptr;
        CREATE_HIP(hipHostGetDevicePointer(&dp, c->host_pin, 0));
        if (!dp) return bail(SSN_E_HIP);
        double *pin_dev = (double *)dp;
        c->f_host_dev = pin_dev + 256;
        c->f_ticket = (unsigned long long *)(c->host_pin + 257);
        *c->f_ticket = 0;
        c->f_ticket_dev = (unsigned long long *)(c->f_host_dev + 1);
        c->pub_host = c->host_pin + 128;                             // bytes 1024..2047
        c->pub_dev = pin_dev + 128;
    }
    if (d->layout == SSN_DENSE_ROWMAJOR) {
        const int64_t nft = (d->p + 63) / 64;
        c->max_chunks = (int)(((int64_t)c->num_cus * xtu_waves_per_cu(d->p) + nft - 1) / nft);
        RowsArgs probe = rows_base(c);
        probe.nrows = (int64_t)1 << 40;
        probe.mode = ROW_GRAD;                                 // the family that writes partials
        const char *force = getenv("SSN_DENSE_PATH");          // "split" forces the two-kernel path
        c->binary = binary_path(d);
        if (c->binary) {
            c->KP = 1;                                         // per-row buffers hold one value per row
            if (c->max_chunks < c->num_cus * 8) c->max_chunks = c->num_cus * 8;
        }
        c->fused = !c->binary && dense_fused_supported(d->dtype, probe) && !(force && strcmp(force, "split") == 0);
        if (c->fused) {
            int g = dense_fused_grid(d->dtype, probe, c->num_cus);
            const int gn = dense_narrow_max_grid(d->p, c->num_cus);
            if (gn > g) g = gn;
            if (g > c->max_chunks) c->max_chunks = g;
            // the one-pass kernel reads whole vectors, up to tail_len elements from the start of a row: on the
            // last row that may leave the matrix, so it gets that row as a zero-padded copy
            const int64_t vec = 16 / c->es;
            int64_t len = (d->p + vec - 1) / vec * vec;
            if (d->ldx > len) len = d->ldx;
            if (len > d->p + 1024) len = d->p + 1024;          // no lane starts a load that far behind the last feature
            c->tail_len = (int)len;
            CREATE_HIP(hipMalloc(&c->tail_row, (size_t)len * c->es));
            CREATE_HIP(hipMemsetAsync(c->tail_row, 0, (size_t)len * c->es, c->st));
            CREATE_HIP(hipMemcpyAsync(c->tail_row, (const char *)d->X + (size_t)(d->n - 1) * d->ldx * c->es, (size_t)d->p * c->es,
                                      hipMemcpyDeviceToDevice, c->st));
        }
        c->part_elems = (int64_t)c->max_chunks * d->p * K;
        CREATE_HIP(hipMalloc(&c->part, (size_t)c->part_elems * c->es));
    }

    // per-row buffers for samples of up to n rows, so that no product call has to (re)allocate them; a multiset
    // sample longer than that grows them (ensure_rows)
    {
        const int64_t rows = round_up(d->n, 16);
        CREATE_HIP(hipMalloc(&c->Ubuf, (size_t)rows * (size_t)c->KP * c->es));
        c->U_rows = rows;
        CREATE_HIP(hipMalloc(&c->Pbuf, (size_t)rows * (size_t)c->KP * c->es));
        c->P_rows = rows;
    }

    // validation: one device pass over the labels and, for CSR, over the index arrays
    int32_t bad = 0;
    CREATE_HIP(launch_check_range(d->labels, d->n, 0, d->C, c->int_dev, c->st));
    if (read_int(c, c->int_dev, &bad) != SSN_OK) return bail(SSN_E_HIP);
    if (bad) return bail(SSN_E_BAD_LABEL);
    if (d->layout == SSN_CSR) {
        CREATE_HIP(launch_check_rowptr(d->rowptr, d->n, d->nnz, c->int_dev, c->st));
        if (read_int(c, c->int_dev, &bad) != SSN_OK) return bail(SSN_E_HIP);
        if (bad) return bail(SSN_E_INVALID_ARG);
        if (d->nnz > 0) {
            CREATE_HIP(launch_check_range(d->colidx, d->nnz, 0, d->p, c->int_dev, c->st));
            if (read_int(c, c->int_dev, &bad) != SSN_OK) return bail(SSN_E_HIP);
            if (bad) return bail(SSN_E_BAD_INDEX);
        }
        if (c->K == 1 && d->nnz > 0) {
            const int64_t nwin = (d->nnz + 63) / 64;
            CREATE_HIP(hipMalloc((void **)&c->csr1_rwin, sizeof(int32_t) * nwin));
            CREATE_HIP(hipMalloc(&c->csr1_zrow, c->es * d->n));
            CREATE_HIP(hipMalloc(&c->csr1_zhead, c->es * nwin));
            CREATE_HIP(launch_csr_window_rows(d->rowptr, d->n, d->nnz, c->csr1_rwin, c->st));
        }
    }
#undef CREATE_HIP
    *out = c;
    return SSN_OK;
}

int ssn_set_stream(ssn_ctx *c, void *stream)
{
    if (!c) return SSN_E_INVALID_ARG;
    SSN_HIP(c, hipStreamSynchronize(c->st));
    c->st = (hipStream_t)stream;
    return SSN_OK;
}

int ssn_objective(ssn_ctx *c, const void *W, double *f)
{
    if (!c || !W || !f) return fail(c, SSN_E_INVALID_ARG, "ssn_objective: null argument");
    return objective_impl(c, W, f);
}

int ssn_gradient(ssn_ctx *c, const void *W, void *G, double *f)
{
    if (!c || !W || !G || W == G) return fail(c, SSN_E_INVALID_ARG, "ssn_gradient: null or aliased argument");
    return gradient_impl(c, W, G, f);
}

int ssn_objective_dev(ssn_ctx *c, const void *W, double *f_dev)
{
    if (!c || !W || !f_dev) return fail(c, SSN_E_INVALID_ARG, "ssn_objective_dev: null argument");
    RowsArgs a = rows_base(c);
    a.nrows = c->d.n;
    a.M = W;
    a.mode = ROW_OBJ;
    int nparts = 0;
    SSN_TRY(launch_rows(c, a, &nparts));
    return enqueue_objective_value(c, W, nparts, 0, -1.0, nullptr, f_dev);
}

int ssn_gradient_dev(ssn_ctx *c, const void *W, void *G, double *f_dev)
{
    if (!c || !W || !G || !f_dev || W == G) return fail(c, SSN_E_INVALID_ARG, "ssn_gradient_dev: null or aliased argument");
    return gradient_impl(c, W, G, nullptr, false, nullptr, 0, nullptr, f_dev);
}

int ssn_vec_to_rowmajor(ssn_ctx *c, const void *vec, void *block)
{
    if (!c || !vec || !block || vec == block) return fail(c, SSN_E_INVALID_ARG, "ssn_vec_to_rowmajor: null or aliased argument");
    SSN_HIP(c, launch_vec_layout(c->d.dtype, c->d.p, c->K, (void *)vec, block, c->d.ldw, true, c->st));
    return SSN_OK;
}

int ssn_rowmajor_to_vec(ssn_ctx *c, const void *block, void *vec)
{
    if (!c || !vec || !block || vec == block) return fail(c, SSN_E_INVALID_ARG, "ssn_rowmajor_to_vec: null or aliased argument");
    SSN_HIP(c, launch_vec_layout(c->d.dtype, c->d.p, c->K, vec, (void *)block, c->d.ldw, false, c->st));
    return SSN_OK;
}

// validate: check the sample indices first (one pass and one synchronisation)
// CSR, inside ssn_solve: the column-sorted view (and support) of the sample S, built on the auxiliary stream
static int prebuild_sample_view(ssn_ctx *c, const int32_t *S, int64_t nS)
{
    c->next_ready = false;
    if (!c->st_aux) {
        SSN_HIP(c, hipStreamCreateWithFlags(&c->st_aux, hipStreamNonBlocking));
        SSN_HIP(c, hipEventCreateWithFlags(&c->ev_aux, hipEventDisableTiming));
    }
    SSN_TRY(build_sample_view(c, &c->csc_next, S, nS, c->st_aux, true));
    SSN_HIP(c, hipEventRecord(c->ev_aux, c->st_aux));
    c->next_S = S;
    c->next_nS = nS;
    c->next_ready = true;
    return SSN_OK;
}

static int hess_prepare_impl(ssn_ctx *c, const void *W, const int32_t *S, int64_t nS, bool validate, bool use_prebuilt = false)
{
    c->prepared = false;
    if (validate) {
        int32_t bad = 0;
        SSN_HIP(c, launch_check_range(S, nS, 0, c->d.n, c->int_dev, c->st));
        SSN_TRY(read_int(c, c->int_dev, &bad));
        if (bad) return fail(c, SSN_E_BAD_INDEX, "ssn_hess_prepare: sample index outside [0,n)");
    }
    const int64_t rows = round_up(nS, 16);
    SSN_TRY(ensure_rows(c, &c->Pbuf, &c->P_rows, rows));
    SSN_TRY(ensure_rows(c, &c->Ubuf, &c->U_rows, rows));
    RowsArgs a = rows_base(c);
    a.S = S;
    a.nrows = nS;
    a.M = W;
    a.mode = ROW_PREP;
    a.UP = c->Pbuf;
    SSN_TRY(launch_rows(c, a, nullptr));
    if (!is_dense(c)) {
        if (use_prebuilt && c->next_ready && c->next_S == S && c->next_nS == nS) {
            std::swap(c->csc_samp, c->csc_next);
            SSN_HIP(c, hipStreamWaitEvent(c->st, c->ev_aux, 0));
        } else {
            SSN_TRY(build_sample_view(c, &c->csc_samp, S, nS, c->st, true));
        }
        c->next_ready = false;
    }
    c->S = S;
    c->nS = nS;
    c->prepared = true;
    return SSN_OK;
}

int ssn_gradient_sampled(ssn_ctx *c, const void *W, const int32_t *S, int64_t nS, void *G, double *f_S)
{
    if (!c || !W || !G || !S || nS < 1 || W == G)
        return fail(c, SSN_E_INVALID_ARG, "ssn_gradient_sampled: null or aliased argument, or nS < 1");
    int32_t bad = 0;
    SSN_HIP(c, launch_check_range(S, nS, 0, c->d.n, c->int_dev, c->st));
    SSN_TRY(read_int(c, c->int_dev, &bad));
    if (bad) return fail(c, SSN_E_BAD_INDEX, "ssn_gradient_sampled: sample index outside [0,n)");
    return gradient_impl(c, W, G, f_S, false, S, nS);
}

int ssn_hess_prepare(ssn_ctx *c, const void *W, const int32_t *S, int64_t nS)
{
    if (!c || !W || !S || nS < 1) return fail(c, SSN_E_INVALID_ARG, "ssn_hess_prepare: null argument or nS < 1");
    return hess_prepare_impl(c, W, S, nS, true);
}

int ssn_hess_apply(ssn_ctx *c, const void *V, void *HV)
{
    if (!c || !V || !HV || V == HV) return fail(c, SSN_E_INVALID_ARG, "ssn_hess_apply: null or aliased argument");
    if (!c->prepared) return fail(c, SSN_E_NOT_PREPARED, "ssn_hess_apply before ssn_hess_prepare");
    return hess_apply_impl(c, V, HV, false, nullptr, nullptr);
}

int ssn_hessvec(ssn_ctx *c, const void *W, const int32_t *S, int64_t nS, const void *V, void *HV)
{
    SSN_TRY(ssn_hess_prepare(c, W, S, nS));
    return ssn_hess_apply(c, V, HV);
}

// every launch of Alg. 2; the final state waits in slots[T]
// n_slope (nullable): on the CSR path the partials of <P_out, G> over the sample's columns are left in red_a,
// *n_slope of them (the rest of the product is CgSlot::pibest * CgSlot::goff); 0 where they are not made
// solve_W / solve_trial / solve_pub (ssn_solve, nullable): on the dense paths with a small block and T > 0 the tail
// launch also forms the slope, the first trial point solve_W + P_out (into solve_trial) and publishes F(x_k), the
// slope and the final state to the host block solve_pub [dev]; *solve_fused tells whether that happened.
static int cg_enqueue(ssn_ctx *c, const void *G, double theta, int32_t T, void *P_out, int *n_slope = nullptr,
                      const void *solve_W = nullptr, void *solve_trial = nullptr, double *solve_pub = nullptr,
                      bool *solve_fused = nullptr)
{
    if (n_slope) *n_slope = 0;
    if (solve_fused) *solve_fused = false;
    if (!c->cg_p) {
        SSN_TRY(vec_bytes_alloc(c, &c->cg_p));
        SSN_TRY(vec_bytes_alloc(c, &c->cg_r));
        SSN_TRY(vec_bytes_alloc(c, &c->cg_s));
    }
    if (is_dense(c) && !c->cg_hs) {
        SSN_TRY(vec_bytes_alloc(c, &c->cg_hs));
        SSN_HIP(c, hipMalloc((void **)&c->cg_parts, sizeof(double) * 4 * RED_MAX_PARTS));
    }
    if (c->slots_cap < T + 1) {
        SSN_HIP(c, hipStreamSynchronize(c->st));
        if (c->slots) (void)hipFree(c->slots);
        if (c->trace_dev) (void)hipFree(c->trace_dev);
        c->slots = nullptr;
        c->trace_dev = nullptr;
        SSN_HIP(c, hipMalloc((void **)&c->slots, sizeof(CgSlot) * (size_t)(T + 1)));
        SSN_HIP(c, hipMalloc((void **)&c->trace_dev, sizeof(double) * 3 * (size_t)(T + 1)));
        SSN_HIP(c, hipMemsetAsync(c->slots, 0, sizeof(CgSlot) * (size_t)(T + 1), c->st));
        c->slots_cap = T + 1;
    }
    CgVecs v{};
    v.p = c->d.p;
    v.K = c->K;
    v.ld = c->d.ldw;
    v.G = G;
    v.pv = c->cg_p;
    v.r = c->cg_r;
    v.s = c->cg_s;
    v.pbest = P_out;
    int vb = vec_blocks(c->d.p * (int64_t)c->K);
    c->cg_gg_parts = 0;
    // one block does it all only where each thread has a handful of elements: a single block walking thousands of
    // elements is a chain of dependent round trips and loses more than the launches it saves
    const bool small = c->d.p * (int64_t)c->K <= 8 * VEC_BLOCK;
    if (is_dense(c) && small) {
        SSN_HIP(c, launch_cg_init_small(c->d.dtype, v, c->slots, c->st));
    } else if (is_dense(c)) {
        SSN_HIP(c, launch_cg_init(c->d.dtype, v, c->red_a, c->red_c, vb, c->st));
        // the initial state is one more reduction of g.g: product 0's finalize does it (no launch of its own)
        if (T > 0) c->cg_gg_parts = vb;
        else SSN_HIP(c, launch_cg_init_state(c->red_a, vb, c->slots, c->st));
    } else {
        // CSR: H_S = scale * X_S^T D X_S + lambda I acts as lambda I on every coordinate outside the columns the
        // sample touches, so r, s, p stay multiples of g there (CgSlot::rho, sigma, pi) and the vectors of
        // Alg. 2 are kept on the sample's columns only: a CG iteration moves ncols * K elements per vector
        // instead of p * K.  The direction is expanded to all coordinates at the end.
        const CscView &sv = c->csc_samp;
        if (!sv.has_support) return fail(c, SSN_E_NOT_PREPARED, "internal: sample view without its support");
        const int64_t need = (int64_t)sv.ncols * c->K;
        if (c->cg_pb_cap < need) {
            SSN_HIP(c, hipStreamSynchronize(c->st));
            if (c->cg_pb) (void)hipFree(c->cg_pb);
            c->cg_pb = nullptr;
            c->cg_pb_cap = 0;
            SSN_HIP(c, hipMalloc(&c->cg_pb, (size_t)(need + need / 8 + 64) * c->es));
            c->cg_pb_cap = need + need / 8 + 64;
        }
        // g.g over all coordinates (red_b) next to g.g over the sample's columns (red_a)
        SSN_HIP(c, launch_dot_part(c->d.dtype, c->d.p, c->K, G, c->d.ldw, G, c->d.ldw, c->red_b, vb, nullptr, c->st));
        const int vb_full = vb;
        v.p = sv.ncols;
        v.ld = c->K;
        v.pbest = c->cg_pb;
        vb = vec_blocks(v.p * (int64_t)c->K);
        SSN_HIP(c, launch_cg_init_support(c->d.dtype, v, G, c->d.ldw, sv.cols, c->red_a, c->red_c, vb, c->st));
        SSN_HIP(c, launch_cg_init_state(c->red_a, vb, c->slots, c->st, c->red_b, vb_full));
    }
    for (int k = 0; k < T; ++k) {
        int n_rr = 0;
        bool p_pending = false;
        SSN_TRY(cg_product_step(c, v, c->slots, k, theta, vb, c->trace_dev, &n_rr, &p_pending));
        if (!is_dense(c))
            SSN_HIP(c, launch_cg_step2(c->d.dtype, v, c->slots + k, c->slots + k + 1, c->red_a, n_rr, theta,
                                       c->trace_dev + 3 * k, c->red_c, p_pending, vb, c->st, c->d.lambda));
    }
    if (is_dense(c) && T > 0) {
        const double *last = c->cg_parts + (size_t)((T - 1) & 1) * 2 * RED_MAX_PARTS;
        if (solve_W && solve_trial && solve_pub && c->d.p * (int64_t)c->K <= OBJ_VALUE_ELEMS) {
            SSN_HIP(c, launch_cg_tail_solve(c->d.dtype, v, c->slots + (T - 1), c->slots + T, last, finalize_blocks(c->d.p, c->K),
                                            theta, c->trace_dev, T, solve_W, solve_trial, c->scal_dev, c->scal_dev + 1,
                                            solve_pub, c->red_a, small ? 1 : vb, c->st));
            if (solve_fused) *solve_fused = true;
        } else {
            SSN_HIP(c, launch_cg_tail(c->d.dtype, v, c->slots + (T - 1), c->slots + T, last, finalize_blocks(c->d.p, c->K),
                                      theta, c->trace_dev, T, vb, c->st));
        }
    }
    if (!is_dense(c)) {
        // the best iterate may still live only in p (it is copied lazily); then all coordinates of the direction
        if (T > 0) SSN_HIP(c, launch_cg_finish(c->d.dtype, v, c->slots + T, vb, c->st));
        SSN_HIP(c, launch_cg_expand(c->d.dtype, c->d.p, c->K, G, c->d.ldw, P_out, c->d.ldw, c->slots + T, c->cg_pb,
                                    c->csc_samp.cols, c->csc_samp.ncols, n_slope ? c->red_a : nullptr, n_slope, c->st));
    }
    return SSN_OK;
}

static void cg_fill_info(const CgSlot &fin, ssn_cg_info *info)
{
    info->iters = fin.iters;
    info->flags = fin.flags;
    info->gnorm = fin.gnorm;
    info->rel_res = fin.gnorm > 0.0 ? fin.rbest / fin.gnorm : 0.0;
}

int ssn_cg(ssn_ctx *c, const void *G, double theta, int32_t T, void *P_out, ssn_cg_info *info, double *trace)
{
    if (!c || !G || !P_out || T < 0 || G == P_out) return fail(c, SSN_E_INVALID_ARG, "ssn_cg: bad argument");
    if (!c->prepared) return fail(c, SSN_E_NOT_PREPARED, "ssn_cg before ssn_hess_prepare");
    SSN_TRY(cg_enqueue(c, G, theta, T, P_out));
    CgSlot fin;
    std::vector<double> tr((size_t)3 * (T > 0 ? T : 1));
    SSN_HIP(c, hipMemcpyAsync(&fin, c->slots + T, sizeof(CgSlot), hipMemcpyDeviceToHost, c->st));
    if (trace && T > 0)
        SSN_HIP(c, hipMemcpyAsync(tr.data(), c->trace_dev, sizeof(double) * 3 * (size_t)T, hipMemcpyDeviceToHost, c->st));
    SSN_HIP(c, hipStreamSynchronize(c->st));
    if (trace)
        for (int k = 0; k < 3 * fin.iters && k < 3 * T; ++k) trace[k] = tr[k];
    if (info) cg_fill_info(fin, info);
    return SSN_OK;
}

int ssn_axpy(ssn_ctx *c, double alpha, const void *P, void *W)
{
    if (!c || !P || !W) return fail(c, SSN_E_INVALID_ARG, "ssn_axpy: null argument");
    SSN_HIP(c, launch_axpy(c->d.dtype, c->d.p, c->K, alpha, P, c->d.ldw, W, c->d.ldw, W, c->d.ldw, c->st));
    return SSN_OK;
}

// <P, G> into scal_dev[1]
static int enqueue_slope(ssn_ctx *c, const void *P, const void *G)
{
    const int vb = vec_blocks(c->d.p * (int64_t)c->K);
    SSN_HIP(c, launch_dot_part(c->d.dtype, c->d.p, c->K, P, c->d.ldw, G, c->d.ldw, c->red_a, vb, nullptr, c->st));
    SSN_HIP(c, launch_combine(c->red_a, vb, 1.0, nullptr, 0, 0.0, c->scal_dev + 1, c->st));
    return SSN_OK;
}

int linesearch_impl(ssn_ctx *c, const void *W, const void *P, double fW, double slope, double beta, double rho,
                    int32_t imax, double *alpha_out, double *f_new, int32_t *n_eval, int32_t *ok, void *G_first = nullptr,
                    const double *first_f = nullptr, int first_status = SSN_OK, void *trial_dst = nullptr,
                    bool margin_cache = true);

int ssn_linesearch(ssn_ctx *c, const void *W, const void *P, const void *G, double fW, double beta, double rho,
                   int32_t imax, double *alpha_out, double *f_new, int32_t *n_eval, int32_t *ok)
{
    if (!c || !W || !P || !G || !alpha_out || !f_new) return fail(c, SSN_E_INVALID_ARG, "ssn_linesearch: null argument");
    double slope = 0.0;
    SSN_TRY(enqueue_slope(c, P, G));
    SSN_TRY(read_scalar(c, c->scal_dev + 1, &slope));
    return linesearch_impl(c, W, P, fW, slope, beta, rho, imax, alpha_out, f_new, n_eval, ok);
}

// The trial point W + alpha P into c->trial and F there enqueued (into scal_dev[0]; *mirrored: also into the
// host-visible word).  G_first (nullable): evaluate with the gradient pass, which leaves grad F there too.
// formed: dst already holds the trial point (the CG tail of ssn_solve wrote it).  dst == nullptr: c->trial.
int trial_enqueue(ssn_ctx *c, const void *W, const void *P, double alpha, void *G_first, bool *mirrored, bool formed = false,
                  void *dst = nullptr)
{
    if (!dst) {
        if (!c->trial) SSN_TRY(vec_bytes_alloc(c, &c->trial));
        dst = c->trial;
    }
    c->sq_for = nullptr;
    if (formed) {
    } else if (c->d.p * (int64_t)c->K > OBJ_VALUE_ELEMS) {
        // a large block: ||trial||^2 for the regulariser comes out of the pass that writes the trial point
        const int vb = vec_blocks(c->d.p * (int64_t)c->K);
        SSN_HIP(c, launch_axpy_sq(c->d.dtype, c->d.p, c->K, alpha, P, c->d.ldw, W, c->d.ldw, dst, c->d.ldw, c->red_sq, vb,
                                  c->st));
        c->sq_for = dst;
        c->n_sq = vb;
    } else {
        SSN_HIP(c, launch_axpy(c->d.dtype, c->d.p, c->K, alpha, P, c->d.ldw, W, c->d.ldw, dst, c->d.ldw, c->st));
    }
    if (G_first) return gradient_impl(c, dst, G_first, nullptr, true, nullptr, 0, mirrored);
    return objective_enqueue(c, dst, mirrored);
}

// The trials of Alg. 3 on cached margins: X (W + alpha P) = X W + alpha X P, so after ONE pass over the data that
// leaves Z = [X W | X P] (n rows of 2K numbers) every trial is a pass over Z; the regulariser of the trial point
// comes from W.W, W.P and P.P.  The same F(W + alpha P) up to rounding (the margins are formed as a sum of two
// products instead of one).  Served: every layout; dense matrices with more than 16 weight columns (two class
// tiles per operand) keep the plain trials.
bool margin_cache_ok(const ssn_ctx *c) { return !is_dense(c) || c->binary || 2 * c->K <= 32; }

int margins_enqueue(ssn_ctx *c, const void *W, const void *P)
{
    if (!c->Zbuf) {
        SSN_HIP(c, hipMalloc(&c->Zbuf, (size_t)c->d.n * (size_t)(2 * c->K) * c->es));
        SSN_HIP(c, hipMalloc((void **)&c->ls_dots, sizeof(double) * 3 * RED_MAX_PARTS));
    }
    RowsArgs a = rows_base(c);
    a.nrows = c->d.n;
    a.M = W;
    a.M2 = P;
    a.mode = ROW_MARGIN;
    a.UP = c->Zbuf;
    a.KP = 2 * c->K;
    SSN_TRY(launch_rows(c, a, nullptr));
    const int vb = vec_blocks(c->d.p * (int64_t)c->K);
    SSN_HIP(c, launch_dot3_part(c->d.dtype, c->d.p, c->K, W, c->d.ldw, P, c->d.ldw, c->ls_dots, vb, c->st));
    return SSN_OK;
}

// F(W + alpha P) from the cached margins into scal_dev[0] and the host-visible word
int cached_trial_enqueue(ssn_ctx *c, double alpha)
{
    int64_t b = (c->d.n + VEC_BLOCK - 1) / VEC_BLOCK;
    if (b > RED_MAX_PARTS) b = RED_MAX_PARTS;
    SSN_HIP(c, launch_ls_trial(c->d.dtype, c->Zbuf, 2 * c->K, c->d.n, c->K, c->d.labels, alpha, c->loss_part, (int)b, c->st));
    const int vb = vec_blocks(c->d.p * (int64_t)c->K);
    SSN_HIP(c, launch_ls_value(c->loss_part, (int)b, scale_full(c), c->ls_dots, vb, alpha, 0.5 * c->d.lambda, c->scal_dev,
                               c->f_host_dev, c->f_ticket_dev, ++c->f_seq, c->st));
    return SSN_OK;
}

// Alg. 3 with the slope <P, G> already on the host.  G_first (nullable): the first trial, alpha = 1, is
// evaluated by the gradient pass, which leaves grad f(W + P) there next to the same F(W + P); when that
// trial is accepted the caller already holds the gradient of the next iterate.  first_f (nullable): the
// caller has already evaluated the first trial (trial_enqueue + read_objective): its value and status.
// On return the trial buffer (trial_dst, or c->trial) holds W + alpha P for the alpha returned: the last point
// evaluated is the one the caller moves to, whether the Armijo test held there or the reductions ran out.
int linesearch_impl(ssn_ctx *c, const void *W, const void *P, double fW, double slope, double beta, double rho,
                    int32_t imax, double *alpha_out, double *f_new, int32_t *n_eval, int32_t *ok, void *G_first,
                    const double *first_f, int first_status, void *trial_dst, bool margin_cache)
{
    double alpha = 1.0, ft = 0.0;
    int i = 0, evals = 0, good = 0;
    // trials this function evaluates itself go through the cached margins (the first of them pays for the pass that
    // fills the cache); a first trial the caller asked to be evaluated with the gradient pass (G_first) keeps that pass
    const bool cache = margin_cache && margin_cache_ok(c);
    bool cached = false, formed = true;
    for (;;) {
        int s;
        if (i == 0 && first_f) {
            ft = *first_f;
            s = first_status;
        } else if (cache && !(i == 0 && G_first)) {
            if (!cached) SSN_TRY(margins_enqueue(c, W, P));
            cached = true;
            SSN_TRY(cached_trial_enqueue(c, alpha));
            s = read_objective(c, true, &ft);
            formed = false;
        } else {
            bool mirrored = false;
            SSN_TRY(trial_enqueue(c, W, P, alpha, i == 0 ? G_first : nullptr, &mirrored, false, trial_dst));
            s = read_objective(c, mirrored, &ft);
        }
        if (s != SSN_OK && s != SSN_E_NONFINITE) return s;
        ++evals;
        if (s == SSN_OK && !(ft > fW + alpha * beta * slope)) { good = 1; break; }
        if (i > imax) break;
        ++i;
        alpha *= rho;
    }
    if (!formed) {      // the point the caller moves to: W + alpha P for the step returned
        void *dst = trial_dst;
        if (!dst) {
            if (!c->trial) SSN_TRY(vec_bytes_alloc(c, &c->trial));
            dst = c->trial;
        }
        c->sq_for = nullptr;
        SSN_HIP(c, launch_axpy(c->d.dtype, c->d.p, c->K, alpha, P, c->d.ldw, W, c->d.ldw, dst, c->d.ldw, c->st));
    }
    *alpha_out = alpha;
    *f_new = ft;
    if (n_eval) *n_eval = evals;
    if (ok) *ok = good;
    return SSN_OK;
}

int ssn_predict(ssn_ctx *c, const void *W, int32_t *pred, double *acc)
{
    if (!c || !W) return fail(c, SSN_E_INVALID_ARG, "ssn_predict: null argument");
    RowsArgs a = rows_base(c);
    a.nrows = c->d.n;
    a.M = W;
    a.mode = ROW_PRED;
    a.pred = pred;
    int nparts = 0;
    SSN_TRY(launch_rows(c, a, &nparts));
    if (acc) {
        int32_t hits = 0;
        SSN_HIP(c, launch_sum_int(c->hit_part, nparts, c->int_dev + 1, c->st));
        SSN_TRY(read_int(c, c->int_dev + 1, &hits));
        *acc = (double)hits / (double)c->d.n;
    }
    return SSN_OK;
}

int ssn_accuracy(ssn_ctx *c, const ssn_desc *test, const void *W, double *acc)
{
    if (!c || !test || !W || !acc) return fail(c, SSN_E_INVALID_ARG, "ssn_accuracy: null argument");
    if (test->p != c->d.p || test->C != c->d.C || test->dtype != c->d.dtype || test->ldw != c->d.ldw)
        return fail(c, SSN_E_INVALID_ARG, "ssn_accuracy: the held-out rows must share p, C, dtype and ldw with the context");
    // the held-out rows get a context of their own for the duration of the call (labels and indices validated as
    // at ssn_create), on the caller's stream: W is then ordered behind whatever the context has enqueued
    ssn_desc td = *test;
    td.stream = (void *)c->st;
    ssn_ctx *t = nullptr;
    const int s = ssn_create(&t, &td);
    if (s != SSN_OK) return fail(c, s, "ssn_accuracy: the description of the held-out rows was rejected");
    const int r = ssn_predict(t, W, nullptr, acc);
    if (r != SSN_OK) c->err = "ssn_accuracy: " + t->err;
    ssn_destroy(t);
    return r;
}

int ssn_solve(ssn_ctx *c, void *W, const ssn_params *pr, ssn_iter_record *log, int32_t max_log, int32_t *iters_done)
{
    if (!c || !W || !pr || !pr->S_all || pr->nS < 1 || pr->iters < 0)
        return fail(c, SSN_E_INVALID_ARG, "ssn_solve: bad argument");
    if (!c->grad) SSN_TRY(vec_bytes_alloc(c, &c->grad));
    if (!c->dir) SSN_TRY(vec_bytes_alloc(c, &c->dir));
    if (!c->trial) SSN_TRY(vec_bytes_alloc(c, &c->trial));
    if (pr->Sg_all && pr->nSg < 1) return fail(c, SSN_E_INVALID_ARG, "ssn_solve: gradient sample size < 1");
    // the whole sample schedule is checked once, not sample by sample
    if (pr->iters > 0) {
        int32_t bad = 0;
        SSN_HIP(c, launch_check_range(pr->S_all, (int64_t)pr->iters * pr->nS, 0, c->d.n, c->int_dev, c->st));
        SSN_TRY(read_int(c, c->int_dev, &bad));
        if (bad) return fail(c, SSN_E_BAD_INDEX, "ssn_solve: sample index outside [0,n)");
        if (pr->Sg_all) {
            SSN_HIP(c, launch_check_range(pr->Sg_all, (int64_t)pr->iters * pr->nSg, 0, c->d.n, c->int_dev, c->st));
            SSN_TRY(read_int(c, c->int_dev, &bad));
            if (bad) return fail(c, SSN_E_BAD_INDEX, "ssn_solve: gradient sample index outside [0,n)");
        }
    }
    // sub-sampled gradient: no pass over all rows produces F(x_k); it is evaluated once here and then
    // carried over from the accepted line-search trial
    double f_carry = 0.0;
    if (pr->Sg_all && pr->iters > 0) SSN_TRY(objective_impl(c, W, &f_carry));
    // Look-ahead (full gradient only): a Newton-type step is accepted at alpha = 1 most of the time, and the
    // accepted trial point is the next iterate.  So the first trial of the line search is evaluated by the
    // gradient pass (F and grad F from one read of the data), and when it is accepted the next iteration
    // starts with its gradient in hand: one pass over the data less per iteration, the same numbers.  After
    // a rejected first trial the plain objective pass is used until a first trial is accepted again.
    const bool look = !pr->Sg_all && !(pr->flags & SSN_SOLVE_NO_LOOKAHEAD);
    if (look && !c->grad_next) SSN_TRY(vec_bytes_alloc(c, &c->grad_next));
    bool look_on = look, have_next = false;
    double f_next = 0.0;
    // Phase times come from events on the stream (six records per iteration; SSN_SOLVE_NO_PHASE_TIMES leaves
    // them out).  The host waits for the device once per iteration -- f, |g|, the slope, the CG state and the
    // first line-search trial come back together -- plus once per further trial.  The last two phases of an
    // iteration are read one synchronisation later.
    constexpr int NE = 6;
    const bool timing = !(pr->flags & SSN_SOLVE_NO_PHASE_TIMES);
    hipEvent_t ev[2][NE] = {};
    if (timing)
        for (auto &set : ev)
            for (auto &e : set) SSN_HIP(c, hipEventCreate(&e));
    auto mark = [&](hipEvent_t e) { return timing ? hipEventRecord(e, c->st) : hipSuccess; };
    const int vb = vec_blocks(c->d.p * (int64_t)c->K);
    auto ms_between = [&](hipEvent_t a, hipEvent_t b) {
        float t = 0.f;
        return hipEventElapsedTime(&t, a, b) == hipSuccess ? (double)t : std::nan("");
    };
    int status = SSN_OK;
    int pending = -1;                        // iteration whose line-search / update times are still to be read
    ssn_iter_record pend_rec{};
    auto flush_pending = [&]() {
        if (pending < 0) return;
        hipEvent_t *E = ev[pending & 1];
        pend_rec.ms_linesearch = timing ? ms_between(E[3], E[4]) : std::nan("");
        pend_rec.ms_update = timing ? ms_between(E[4], E[5]) : std::nan("");
        if (log && pending < max_log) log[pending] = pend_rec;
        pending = -1;
    };
    // The iterate lives alternately in the caller's block and in the trial buffer: a step is a change of roles
    // (see the end of the loop), and the caller's block receives the final iterate at the end if it is not there.
    void *cur = W, *oth = c->trial;
    int k = 0;
#define SOLVE_TRY(expr)                     \
    do {                                    \
        status = (expr);                    \
        if (status != SSN_OK) goto done;    \
    } while (0)
#define SOLVE_HIP(call)                                                                            \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            c->err = std::string(#call) + ": " + hipGetErrorString(e_);                            \
            status = SSN_E_HIP;                                                                    \
            goto done;                                                                             \
        }                                                                                          \
    } while (0)
    for (; k < pr->iters; ++k) {
        hipEvent_t *E = ev[k & 1];
        ssn_iter_record rec{};
        rec.test_acc = std::nan("");
        SOLVE_HIP(mark(E[0]));
        if (pr->Sg_all) SOLVE_TRY(gradient_impl(c, cur, c->grad, nullptr, false, pr->Sg_all + (int64_t)k * pr->nSg, pr->nSg));
        else if (!have_next) SOLVE_TRY(gradient_impl(c, cur, c->grad, nullptr, true));
        SOLVE_HIP(mark(E[1]));
        SOLVE_TRY(hess_prepare_impl(c, cur, pr->S_all + (int64_t)k * pr->nS, pr->nS, false, true));
        SOLVE_HIP(mark(E[2]));
        // CSR: CG leaves the slope's partials (n_slope > 0)
        int n_slope = 0;
        bool tail_fused = false;             // small dense blocks: the CG tail has formed slope, trial point and publication
        SOLVE_TRY(cg_enqueue(c, c->grad, pr->theta, pr->T, c->dir, &n_slope, cur, oth, c->pub_dev, &tail_fused));
        // F(x_k), <dir, g> and the final CG state (which carries ||g||) reach the host through host-visible
        // memory written by one small kernel
        if (n_slope == 0 && !tail_fused)
            SOLVE_HIP(launch_dot_part(c->d.dtype, c->d.p, c->K, c->dir, c->d.ldw, c->grad, c->d.ldw, c->red_a, vb, nullptr,
                                      c->st));
        const double *pub = c->pub_host;
        if (!tail_fused)
            SOLVE_HIP(launch_solve_publish(c->red_a, n_slope ? n_slope : vb, c->scal_dev, c->slots + pr->T, c->scal_dev + 1,
                                           c->pub_dev, n_slope > 0, c->st));
        SOLVE_HIP(mark(E[3]));
        // The first trial of the line search is x_k + dir whatever the host reads back, so it is enqueued
        // before the host waits: one wait per iteration covers the CG results and the trial's F.
        const bool ahead = look_on && k + 1 < pr->iters;
        bool first_mirrored = false;
        SOLVE_TRY(trial_enqueue(c, cur, c->dir, 1.0, ahead ? c->grad_next : nullptr, &first_mirrored, tail_fused, oth));
        // CSR: while the device works through the queue above, the view of the next sample is built beside it
        if (!is_dense(c) && k + 1 < pr->iters) SOLVE_TRY(prebuild_sample_view(c, pr->S_all + (int64_t)(k + 1) * pr->nS, pr->nS));
        double f_first = 0.0;
        const int first_status = read_objective(c, first_mirrored, &f_first);       // the one wait of the iteration
        if (first_status != SSN_OK && first_status != SSN_E_NONFINITE) {
            status = first_status;
            goto done;
        }
        flush_pending();
        {
            rec.f = pr->Sg_all ? f_carry : (have_next ? f_next : pub[0]);
            const double slope = pub[1];
            CgSlot fin;
            memcpy(&fin, pub + 2, sizeof(CgSlot));
            rec.gnorm = fin.gnorm;
            if (timing) {
                rec.ms_grad = ms_between(E[0], E[1]);
                rec.ms_prepare = ms_between(E[1], E[2]);
                rec.ms_cg = ms_between(E[2], E[3]);
            }
            if (!std::isfinite(rec.f)) {
                status = fail(c, SSN_E_NONFINITE, "objective is not finite");
                goto done;
            }
            if (rec.gnorm < pr->eps) {       // converged: the direction and the trial computed above are discarded
                rec.ms_prepare = rec.ms_cg = timing ? 0.0 : std::nan("");
                if (log && k < max_log) log[k] = rec;
                break;
            }
            ssn_cg_info info{};
            cg_fill_info(fin, &info);
            rec.cg_iters = info.iters;
            rec.cg_rel_res = info.rel_res;
            double fn = 0.0;
            SOLVE_TRY(linesearch_impl(c, cur, c->dir, rec.f, slope, pr->beta, pr->rho, pr->imax, &rec.alpha, &fn, &rec.ls_evals,
                                      &rec.ls_ok, nullptr, &f_first, first_status, oth, !(pr->flags & SSN_SOLVE_NO_MARGIN_CACHE)));
            f_carry = fn;
            const bool first_accepted = rec.ls_ok && rec.ls_evals == 1;
            have_next = ahead && first_accepted;
            if (have_next) {
                std::swap(c->grad, c->grad_next);
                f_next = fn;
            }
            look_on = look && first_accepted;
        }
        SOLVE_HIP(mark(E[4]));
        // line 7 of Alg. 1, x_{k+1} = x_k + alpha p_k: the trial buffer already holds exactly that (the last point
        // the line search evaluated, formed by the same arithmetic), so the two buffers change roles
        std::swap(cur, oth);
        if (pr->test) {
            // the held-out context runs on its own stream: wait for the update first
            SOLVE_HIP(hipStreamSynchronize(c->st));
            SOLVE_TRY(ssn_predict(pr->test, cur, nullptr, &rec.test_acc));
        }
        SOLVE_HIP(mark(E[5]));
        pending = k;
        pend_rec = rec;
    }
done:
#undef SOLVE_TRY
#undef SOLVE_HIP
    if (cur != W) {                          // the final iterate into the caller's block
        const hipError_t ce = launch_scale_copy(c->d.dtype, c->d.p, c->K, 1.0, cur, c->d.ldw, W, c->d.ldw, nullptr, c->st);
        if (ce != hipSuccess && status == SSN_OK) {
            c->err = std::string("copy of the final iterate: ") + hipGetErrorString(ce);
            status = SSN_E_HIP;
        }
    }
    (void)hipStreamSynchronize(c->st);
    if (c->st_aux) (void)hipStreamSynchronize(c->st_aux);
    c->next_ready = false;                   // a view built ahead is only good inside this call
    flush_pending();
    if (timing)
        for (auto &set : ev)
            for (auto &e : set) (void)hipEventDestroy(e);
    if (iters_done) *iters_done = k;
    return status;
}

}  // extern "C"

// ---- ssn_hessvec_static: the product for callers that cannot allocate --------------------------------------
// Its workspace is this array in the library's device image.  The name below is a host-side stand-in, not a
// device address: host code uses the address hipGetSymbolAddress returns for the current device (each GPU holds
// its own copy of the array), looked up once per device and kept in static_dev[].
static __device__ __align__(256) unsigned char scratch[SSN_STATIC_WORKSPACE_BYTES];

namespace {
struct StaticDev {
    unsigned char *ptr = nullptr;     // device address of `scratch` on this GPU
    int num_cus = 0;
};
constexpr int STATIC_MAX_DEVICES = 64;
StaticDev static_dev[STATIC_MAX_DEVICES];
std::mutex static_mu;

// first call on a device (that device current): the array's address there and the device's compute-unit count
int static_setup(int dev, StaticDev *out)
{
    std::lock_guard<std::mutex> lock(static_mu);
    StaticDev &sd = static_dev[dev];
    if (!sd.ptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SSN_E_HIP;
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return SSN_E_HIP;
        sd.num_cus = cus;
        sd.ptr = (unsigned char *)ptr;
    }
    *out = sd;
    return SSN_OK;
}
}  // namespace

extern "C" int ssn_hessvec_static(const ssn_desc *d, const void *W, const int32_t *S, int64_t nS, const void *V, void *HV)
{
    if (!d || !W || !S || !V || !HV || nS < 1 || V == HV || W == HV) return SSN_E_INVALID_ARG;
    if (d->n < 1 || d->p < 1 || d->C < 2 || !(d->lambda >= 0.0)) return SSN_E_INVALID_ARG;
    if (d->dtype != SSN_F32 && d->dtype != SSN_F64) return SSN_E_INVALID_ARG;
    if (d->scale != SSN_SCALE_MEAN && d->scale != SSN_SCALE_SUM) return SSN_E_INVALID_ARG;
    if (d->layout == SSN_CSR) return SSN_E_UNSUPPORTED;          // its column-sorted view is built with allocations
    if (d->layout != SSN_DENSE_ROWMAJOR) return SSN_E_INVALID_ARG;
    const int K = d->C - 1;
    if (!d->X || d->ldx < d->p || d->ldw < K) return SSN_E_INVALID_ARG;
    if (K > 32 || d->n >= (int64_t)1 << 31 || d->p >= (int64_t)1 << 31 || nS >= (int64_t)1 << 31) return SSN_E_UNSUPPORTED;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return SSN_E_HIP;
    StaticDev sd;
    SSN_TRY(static_setup(dev, &sd));

    // a context on the stack whose workspace pointers are carved out of the fixed array: the entry points' own
    // code paths then run unchanged (same kernels, same grids as ssn_hessvec on a created context)
    ssn_ctx c;
    c.d = *d;
    c.K = K;
    c.es = d->dtype == SSN_F32 ? 4 : 8;
    c.KP = (K + 15) / 16 * 16;
    c.st = (hipStream_t)d->stream;
    c.num_cus = sd.num_cus;
    c.wave_parts = c.num_cus * 16 * ROWS_WAVES_PER_BLOCK;
    const int64_t rows = round_up(nS, 16);
    RowsArgs probe = rows_base(&c);
    probe.nrows = nS;
    probe.mode = ROW_APPLY;
    const char *force = getenv("SSN_DENSE_PATH");
    c.binary = binary_path(d);
    if (c.binary) c.KP = 1;
    c.fused = !c.binary && dense_fused_supported(d->dtype, probe) && !(force && strcmp(force, "split") == 0);
    if (c.binary) {
        c.max_chunks = (int)(rows / 8 < (int64_t)c.num_cus * 8 ? rows / 8 : (int64_t)c.num_cus * 8);
    } else if (c.fused) {
        c.max_chunks = dense_fused_grid(d->dtype, probe, c.num_cus);
        probe.mode = ROW_PREP;                 // writes no partials, but its grid is checked against the same bound
        const int gp = dense_fused_grid(d->dtype, probe, c.num_cus);
        if (gp > c.max_chunks) c.max_chunks = gp;
        const int64_t vec = 16 / c.es;
        int64_t len = (d->p + vec - 1) / vec * vec;
        if (d->ldx > len) len = d->ldx;
        if (len > d->p + 1024) len = d->p + 1024;
        c.tail_len = (int)len;
    } else {
        const int64_t nft = (d->p + 63) / 64;
        int64_t mc = ((int64_t)c.num_cus * xtu_waves_per_cu(d->p) + nft - 1) / nft;
        if (mc > rows / 16) mc = rows / 16;
        c.max_chunks = (int)mc;
    }
    // layout of the workspace (every piece 256-byte aligned)
    size_t off = 0;
    auto carve = [&](size_t bytes) {
        unsigned char *q = sd.ptr + off;
        off += (bytes + 255) / 256 * 256;
        return (void *)q;
    };
    const size_t row_bytes = (size_t)rows * (size_t)c.KP * c.es;
    const size_t part_bytes = (size_t)c.max_chunks * (size_t)d->p * (size_t)K * c.es;
    const size_t need = round_up(sizeof(double) * c.wave_parts, 256) + round_up((int64_t)c.tail_len * (int64_t)c.es, 256)
                        + 2 * round_up((int64_t)row_bytes, 256) + round_up((int64_t)part_bytes, 256);
    if (need > (size_t)SSN_STATIC_WORKSPACE_BYTES) return SSN_E_TOO_LARGE;
    c.loss_part = (double *)carve(sizeof(double) * c.wave_parts);
    if (c.fused) c.tail_row = carve((size_t)c.tail_len * c.es);
    c.Pbuf = carve(row_bytes);
    c.P_rows = rows;
    c.Ubuf = carve(row_bytes);
    c.U_rows = rows;
    c.part = carve(part_bytes);
    c.part_elems = (int64_t)c.max_chunks * d->p * K;
    if (c.fused)      // zero-padded copy of the last row (a kernel, not a memset: the call may be under graph capture)
        SSN_HIP(&c, launch_pad_copy(d->dtype, (const char *)d->X + (size_t)(d->n - 1) * d->ldx * c.es, d->p, c.tail_row,
                                    c.tail_len, c.st));
    SSN_TRY(hess_prepare_impl(&c, W, S, nS, false));
    return hess_apply_impl(&c, V, HV, false, nullptr, nullptr);
}

extern "C" {

int ssn_time_kernel(ssn_ctx *c, int32_t which, const void *M, int32_t reps, double *ms)
{
    if (!c || !M || !ms || reps < 1 || which < 0 || which > 5) return fail(c, SSN_E_INVALID_ARG, "ssn_time_kernel: bad argument");
    if (which == 5) {
        // plain streaming read of the data matrix (dense: n*ldx elements; CSR: the value array)
        const void *src = is_dense(c) ? c->d.X : c->d.vals;
        int64_t bytes = (is_dense(c) ? c->d.n * c->d.ldx : c->d.nnz) * (int64_t)c->es;
        bytes -= bytes % 16;
        if (!src || bytes < 16 || (uintptr_t)src % 16) return fail(c, SSN_E_INVALID_ARG, "ssn_time_kernel: buffer not streamable");
        hipEvent_t s0, s1;
        SSN_HIP(c, hipEventCreate(&s0));
        SSN_HIP(c, hipEventCreate(&s1));
        hipError_t e = hipEventRecord(s0, c->st);
        for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch_stream_read(src, bytes, c->loss_part, c->num_cus * 8, c->st);
        if (e == hipSuccess) e = hipEventRecord(s1, c->st);
        if (e == hipSuccess) e = hipEventSynchronize(s1);
        float tt = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&tt, s0, s1);
        (void)hipEventDestroy(s0);
        (void)hipEventDestroy(s1);
        SSN_HIP(c, e);
        *ms = (double)tt / reps;
        return SSN_OK;
    }
    const bool sampled = which >= 3;
    if (sampled && !c->prepared) return fail(c, SSN_E_NOT_PREPARED, "ssn_time_kernel: no prepared sample");
    const int64_t nrows = sampled ? c->nS : c->d.n;
    SSN_TRY(ensure_rows(c, &c->Ubuf, &c->U_rows, round_up(nrows, 16)));
    RowsArgs a = rows_base(c);
    a.S = sampled ? c->S : nullptr;
    a.nrows = nrows;
    a.M = M;
    a.UP = c->Ubuf;
    a.Pin = c->Pbuf;
    a.mode = which == 0 ? ROW_OBJ : (which == 1 ? ROW_GRAD : ROW_APPLY);
    a.part = c->part;
    XtuArgs x = xtu_base(c);
    x.S = a.S;
    x.nrows = nrows;
    x.U = c->Ubuf;
    if (is_dense(c)) choose_chunks(c, nrows, &x.rows_per_chunk, &x.nchunks);
    if (which == 4 && is_dense(c) && !c->fused) xtu_after_apply(c, &x);      // as the last which = 3 launch left it
    if ((!is_dense(c) || c->fused) && (which == 2 || which == 4) && !c->trial) SSN_TRY(vec_bytes_alloc(c, &c->trial));
    const int fused_parts = c->fused ? dense_fused_grid(c->d.dtype, a, c->num_cus) : 0;
    hipEvent_t e0, e1;
    SSN_HIP(c, hipEventCreate(&e0));
    SSN_HIP(c, hipEventCreate(&e1));
    int status = SSN_OK;
    hipError_t he = hipEventRecord(e0, c->st);
    for (int r = 0; r < reps && status == SSN_OK && he == hipSuccess; ++r) {
        if (which == 2 || which == 4) {
            if (c->fused) status = finalize_dense(c, fused_parts, sampled ? scale_sample(c) : scale_full(c), M, c->trial, false, nullptr, nullptr);
            else if (is_dense(c)) he = launch_xtu(c, x);
            else {
                const CscView *view = nullptr;
                status = csc_view_for(c, a.S, &view);
                if (status == SSN_OK)
                    he = launch_csc_apply(c->d.dtype, *view, c->K, c->KP, c->Ubuf, sampled ? scale_sample(c) : scale_full(c),
                                          c->trial, c->d.ldw, nullptr, nullptr, c->st);
            }
        } else {
            status = launch_rows(c, a, nullptr);
        }
    }
    if (he == hipSuccess) he = hipEventRecord(e1, c->st);
    if (he == hipSuccess) he = hipEventSynchronize(e1);
    float t = 0.f;
    if (he == hipSuccess) he = hipEventElapsedTime(&t, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (status != SSN_OK) return status;
    SSN_HIP(c, he);
    *ms = (double)t / reps;
    return SSN_OK;
}

int ssn_sampled_slices(const ssn_ctx *c)
{
    if (!c) return SSN_E_INVALID_ARG;
    return c->z_active ? c->z_slices : 0;
}

int ssn_dense_path(const ssn_ctx *c)
{
    if (!c) return SSN_E_INVALID_ARG;
    if (!is_dense(c)) return 0;
    if (c->binary) return 3;
    return c->fused ? 2 : 1;
}

}  // extern "C"
