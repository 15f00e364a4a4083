// Column-sorted view of a set of CSR rows and the transposed product X_rows^T U on it.
//
// The transposed product of eq. (13) / Alg. 6 adds x_ij * u_i into row j of the result for every stored
// entry.  Scattering from the CSR rows would need floating-point atomics (an order of summation that
// changes from run to run); instead the entries of the selected rows are kept sorted by column -- the
// whole matrix is sorted once, when the context first needs it, and a sample's list is filtered out of
// that at every ssn_hess_prepare -- and each product then GATHERS: the entries of a column are
// consecutive, rows of U are read, and every result element has exactly one writer and one order of
// summation.
//
// Work is cut into pieces: a piece ends where the column changes and at every PIECE_LEN-th entry, so hot
// columns (a few appear in almost every row of text-like data) are spread over many lane groups.  A
// piece that is a whole column adds into the result directly; the pieces of a longer column leave
// partial sums that a second kernel adds in piece order.
//
// The one-off sort of the whole matrix (and the fallback construction for samples of matrices with very
// uneven row lengths) uses hipCUB's device radix sort and prefix sums; the construction of a sample's
// view from the whole matrix's and the product kernels are hand-written.
#include "ssn_internal.h"
#include "ssn_math.h"

#include <hipcub/hipcub.hpp>

namespace ssn {

constexpr int PIECE_LEN = 64;

// ---- construction ---------------------------------------------------------------------------
__global__ __launch_bounds__(VEC_BLOCK) void csc_row_len_kernel(const int32_t *rowptr, const int32_t *S, int64_t nrows,
                                                                 int32_t *len)
{
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i <= nrows; i += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t r = (i < nrows) ? (S ? (int64_t)S[i] : i) : 0;
        len[i] = (i < nrows) ? rowptr[r + 1] - rowptr[r] : 0;
    }
}

// one wave per selected row: copy its entries to positions off[sv].. with the sample position as payload
template <typename T>
__global__ __launch_bounds__(256) void csc_expand_kernel(const int32_t *rowptr, const int32_t *colidx, const T *vals,
                                                         const int32_t *S, int64_t nrows, const int32_t *off,
                                                         int32_t *key_in, int32_t *idx_in, int32_t *row_in, T *val_in)
{
    const int lane = threadIdx.x & 63;
    const int64_t nw = (int64_t)gridDim.x * 4;
    for (int64_t sv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); sv < nrows; sv += nw) {
        const int64_t r = S ? S[sv] : sv;
        const int64_t b = rowptr[r], e = rowptr[r + 1];
        const int64_t o = off[sv];
        for (int64_t t = b + lane; t < e; t += 64) {
            const int64_t d = o + (t - b);
            key_in[d] = colidx[t];
            idx_in[d] = (int32_t)d;
            row_in[d] = (int32_t)sv;
            val_in[d] = vals[t];
        }
    }
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void csc_permute_kernel(const int32_t *idx, const int32_t *row_in, const T *val_in,
                                                                 int64_t nnz, int32_t *row, T *val)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK) {
        const int32_t e = idx[t];
        row[t] = row_in[e];
        val[t] = val_in[e];
    }
}

// flag[t] = 1 where a piece starts: first entry of a column, or every PIECE_LEN-th entry
__global__ __launch_bounds__(VEC_BLOCK) void csc_piece_flag_kernel(const int32_t *key, int64_t nnz, int32_t *flag)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK)
        flag[t] = (t == 0 || key[t] != key[t - 1] || (t % PIECE_LEN) == 0) ? 1 : 0;
}

// piece_start[k] / piece_col[k]: first entry and column of piece k; piece_start ends with nnz, piece_col with
// four sentinels (-1) so that readers may look a few pieces ahead
__global__ __launch_bounds__(VEC_BLOCK) void csc_piece_start_kernel(const int32_t *flag, const int32_t *pid, const int32_t *key,
                                                                    int64_t nnz, int32_t *piece_start, int32_t *piece_col,
                                                                    int32_t *npieces_out)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK) {
        if (flag[t]) {
            piece_start[pid[t]] = (int32_t)t;
            piece_col[pid[t]] = key[t];
        }
        if (t == nnz - 1) {
            const int32_t np = pid[t] + flag[t];
            piece_start[np] = (int32_t)nnz;
            for (int k = 0; k < 4; ++k) piece_col[np + k] = -1;
            *npieces_out = np;
        }
    }
}

// ---- support of the view: the distinct columns, and the view in their coordinates ----------------------
// head[t] = 1 where a new column starts in the sorted entry list
__global__ __launch_bounds__(VEC_BLOCK) void csc_head_flag_kernel(const int32_t *key, int64_t nnz, int32_t *head)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK)
        head[t] = (t == 0 || key[t] != key[t - 1]) ? 1 : 0;
}

// rank[t] (exclusive scan of head, so rank + head - 1 is the position of entry t's column among the distinct
// columns) -> cols[position] = column; ccol[e] = position for the entry's place e in row order (idx[t]);
// *ncols_out = number of distinct columns
__global__ __launch_bounds__(VEC_BLOCK) void csc_support_kernel(const int32_t *key, const int32_t *head, const int32_t *rank,
                                                                const int32_t *idx, int64_t nnz, int32_t *cols, int32_t *ccol,
                                                                int32_t *ncols_out)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK) {
        const int32_t pos = rank[t] + head[t] - 1;
        if (head[t]) cols[pos] = key[t];
        ccol[idx[t]] = pos;
        if (t == nnz - 1) *ncols_out = pos + 1;
    }
}

// piece_cpos[k] = position of piece k's column among the distinct columns (four sentinels -1 at the end)
__global__ __launch_bounds__(VEC_BLOCK) void csc_piece_cpos_kernel(const int32_t *piece_start, const int32_t *head,
                                                                   const int32_t *rank, int32_t npieces, int32_t *piece_cpos)
{
    for (int64_t k = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; k < npieces + 4; k += (int64_t)gridDim.x * VEC_BLOCK) {
        if (k < npieces) {
            const int32_t t = piece_start[k];
            piece_cpos[k] = rank[t] + head[t] - 1;
        } else {
            piece_cpos[k] = -1;
        }
    }
}

static int grid_for(int64_t n)
{
    int64_t b = (n + VEC_BLOCK - 1) / VEC_BLOCK;
    if (b > 65536) b = 65536;
    if (b < 1) b = 1;
    return (int)b;
}

#define CSC_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return e_;                \
    } while (0)

static hipError_t grow(void **ptr, int64_t *cap, int64_t need, size_t elem)
{
    if (*cap >= need) return hipSuccess;
    if (*ptr) CSC_HIP(hipFree(*ptr));
    *ptr = nullptr;
    *cap = 0;
    const int64_t want = need + need / 8 + 64;
    CSC_HIP(hipMalloc(ptr, (size_t)want * elem));
    *cap = want;
    return hipSuccess;
}

void csc_free(CscView *v)
{
    void *all[] = {v->key, v->row, v->val, v->piece_start, v->piece_col, v->piece_part, v->off, v->key_in, v->idx_in, v->idx_out,
                   v->row_in, v->val_in, v->flag, v->pid, v->cub_tmp, v->count_dev, v->cols, v->ccol, v->piece_cpos,
                   v->cnt, v->head, v->next, v->tsum, v->toff, v->ftoff, v->len, v->bitmap, v->eidx, v->csr_pos, v->win_pid};
    for (void *q : all)
        if (q) (void)hipFree(q);
    *v = CscView{};
}

void csc_free_scratch(CscView *v)
{
    void *all[] = {v->key_in, v->idx_in, v->idx_out, v->row_in, v->val_in, v->flag, v->pid, v->cub_tmp};
    for (void *q : all)
        if (q) (void)hipFree(q);
    v->key_in = v->idx_in = v->idx_out = v->row_in = v->flag = v->pid = nullptr;
    v->val_in = v->cub_tmp = nullptr;
    v->cap_in = v->cap_flag = v->cap_pid = v->cap_valin = 0;
    v->cub_bytes = 0;
}

// Build the view of rows S[0..nrows) (S == nullptr: rows 0..nrows-1) of the CSR matrix.  Synchronises the
// stream twice (entry count and piece count come back to size the buffers).
// support: also list the distinct columns of the view (cols, ncols) and express the selected rows in their
// coordinates: (off, ccol, val_in) is then a CSR matrix of nrows rows and ncols columns, and piece_cpos the
// pieces' columns in the same coordinates.  The construction scratch must be kept for that.
hipError_t csc_build(CscView *v, int dtype, const int32_t *rowptr, const int32_t *colidx, const void *vals,
                     const int32_t *S, int64_t nrows, int64_t p, int K, hipStream_t st, bool support)
{
    const size_t es = dtype == SSN_F32 ? 4 : 8;
    v->nnz = 0;
    v->npieces = 0;
    v->win_npieces = -1;                 // the window index of an earlier build is void
    v->ncols = 0;
    v->has_support = false;
    if (!v->count_dev) CSC_HIP(hipMalloc((void **)&v->count_dev, 4 * sizeof(int32_t)));

    auto cub_need = [&](size_t bytes) -> hipError_t {
        if (bytes <= v->cub_bytes) return hipSuccess;
        if (v->cub_tmp) CSC_HIP(hipFree(v->cub_tmp));
        v->cub_tmp = nullptr;
        v->cub_bytes = 0;
        CSC_HIP(hipMalloc(&v->cub_tmp, bytes + 256));
        v->cub_bytes = bytes + 256;
        return hipSuccess;
    };

    // 1. offsets of the selected rows in the expanded entry list
    CSC_HIP(grow((void **)&v->off, &v->cap_off, nrows + 1, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->flag, &v->cap_flag, nrows + 1, sizeof(int32_t)));     // row lengths, for now
    CSC_HIP(grow((void **)&v->pid, &v->cap_pid, nrows + 1, sizeof(int32_t)));
    hipLaunchKernelGGL(csc_row_len_kernel, dim3(grid_for(nrows + 1)), dim3(VEC_BLOCK), 0, st, rowptr, S, nrows, v->flag);
    size_t bytes = 0;
    CSC_HIP(hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, v->flag, v->off, (int)(nrows + 1), st));
    CSC_HIP(cub_need(bytes));
    bytes = v->cub_bytes;
    CSC_HIP(hipcub::DeviceScan::ExclusiveSum(v->cub_tmp, bytes, v->flag, v->off, (int)(nrows + 1), st));
    int32_t total32 = 0;
    CSC_HIP(hipMemcpyAsync(&total32, v->off + nrows, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    CSC_HIP(hipStreamSynchronize(st));
    const int64_t nnz = total32;
    if (nnz < 0) return hipErrorInvalidValue;          // more than 2^31 entries selected
    if (nnz == 0) {
        v->has_support = support;          // no entries: no columns, every selected row is empty (off is all zero)
        return hipSuccess;
    }

    // 2. expand (column, position, sample row, value), sort by column (stable: rows stay in sample order)
    CSC_HIP(grow((void **)&v->key, &v->cap, nnz, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->row, &v->cap_row, nnz, sizeof(int32_t)));
    CSC_HIP(grow(&v->val, &v->cap_val, nnz, es));
    {
        int64_t c0 = v->cap_in, c1 = v->cap_in, c2 = v->cap_in, c3 = v->cap_in, c4 = v->cap_valin;
        CSC_HIP(grow((void **)&v->key_in, &c0, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->idx_in, &c1, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->idx_out, &c2, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->row_in, &c3, nnz, sizeof(int32_t)));
        CSC_HIP(grow(&v->val_in, &c4, nnz, es));
        v->cap_in = c0;
        v->cap_valin = c4;
    }
    CSC_HIP(grow((void **)&v->flag, &v->cap_flag, nnz, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->pid, &v->cap_pid, nnz, sizeof(int32_t)));
    int64_t eb = (nrows + 3) / 4;
    if (eb > 16384) eb = 16384;
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(csc_expand_kernel<float>, dim3((unsigned)eb), dim3(256), 0, st, rowptr, colidx, (const float *)vals,
                           S, nrows, v->off, v->key_in, v->idx_in, v->row_in, (float *)v->val_in);
    else
        hipLaunchKernelGGL(csc_expand_kernel<double>, dim3((unsigned)eb), dim3(256), 0, st, rowptr, colidx,
                           (const double *)vals, S, nrows, v->off, v->key_in, v->idx_in, v->row_in, (double *)v->val_in);
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < p) ++bits;
    bytes = 0;
    CSC_HIP(hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, v->key_in, v->key, v->idx_in, v->idx_out, (int)nnz, 0, bits, st));
    CSC_HIP(cub_need(bytes));
    bytes = v->cub_bytes;
    CSC_HIP(hipcub::DeviceRadixSort::SortPairs(v->cub_tmp, bytes, v->key_in, v->key, v->idx_in, v->idx_out, (int)nnz, 0, bits,
                                               st));
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(csc_permute_kernel<float>, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->idx_out, v->row_in,
                           (const float *)v->val_in, nnz, v->row, (float *)v->val);
    else
        hipLaunchKernelGGL(csc_permute_kernel<double>, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->idx_out, v->row_in,
                           (const double *)v->val_in, nnz, v->row, (double *)v->val);

    // 3. pieces
    hipLaunchKernelGGL(csc_piece_flag_kernel, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->key, nnz, v->flag);
    bytes = 0;
    CSC_HIP(hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, v->flag, v->pid, (int)nnz, st));
    CSC_HIP(cub_need(bytes));
    bytes = v->cub_bytes;
    CSC_HIP(hipcub::DeviceScan::ExclusiveSum(v->cub_tmp, bytes, v->flag, v->pid, (int)nnz, st));
    // there are at most nnz pieces: size the piece arrays from that bound, before the count is known
    CSC_HIP(grow((void **)&v->piece_start, &v->cap_piece, nnz + 1, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->piece_col, &v->cap_pcol, nnz + 4, sizeof(int32_t)));
    hipLaunchKernelGGL(csc_piece_start_kernel, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->flag, v->pid, v->key, nnz,
                       v->piece_start, v->piece_col, v->count_dev);
    if (support) {
        // key_in / idx_in are free once the sort is done: they take the column-head flags and their scan
        CSC_HIP(grow((void **)&v->cols, &v->cap_cols, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->ccol, &v->cap_ccol, nnz, sizeof(int32_t)));
        hipLaunchKernelGGL(csc_head_flag_kernel, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->key, nnz, v->key_in);
        bytes = 0;
        CSC_HIP(hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, v->key_in, v->idx_in, (int)nnz, st));
        CSC_HIP(cub_need(bytes));
        bytes = v->cub_bytes;
        CSC_HIP(hipcub::DeviceScan::ExclusiveSum(v->cub_tmp, bytes, v->key_in, v->idx_in, (int)nnz, st));
        hipLaunchKernelGGL(csc_support_kernel, dim3(grid_for(nnz)), dim3(VEC_BLOCK), 0, st, v->key, v->key_in, v->idx_in,
                           v->idx_out, nnz, v->cols, v->ccol, v->count_dev + 1);
    }
    int32_t counts[2] = {0, 0};
    CSC_HIP(hipMemcpyAsync(counts, v->count_dev, (support ? 2 : 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    CSC_HIP(hipStreamSynchronize(st));
    const int32_t np = counts[0];
    CSC_HIP(grow(&v->piece_part, &v->cap_part, (int64_t)np * K * 2, es));       // piece sums, then run sums
    if (support) {
        CSC_HIP(grow((void **)&v->piece_cpos, &v->cap_pcpos, (int64_t)np + 4, sizeof(int32_t)));
        hipLaunchKernelGGL(csc_piece_cpos_kernel, dim3(grid_for((int64_t)np + 4)), dim3(VEC_BLOCK), 0, st, v->piece_start,
                           v->key_in, v->idx_in, np, v->piece_cpos);
        v->ncols = counts[1];
        v->has_support = true;
    }
    CSC_HIP(hipGetLastError());
    v->nnz = nnz;
    v->npieces = np;
    v->nrows = nrows;
    return hipSuccess;
}

// ---- the view of a sample, filtered out of the whole matrix's view -------------------------------------
// The whole matrix's entries are already sorted by (column, row).  A sample's view is the sub-list of the entries
// whose row is sampled (an entry of a row sampled m times appears m times), in the same order: no sort, one
// counting pass and one copying pass over the whole view's row indices (4 bytes per stored entry) and prefix sums
// written here.  Equal rows of a sample have equal rows of U, so the order of their entries inside a column does
// not change any sum.

constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = VEC_BLOCK * SCAN_ITEMS;

// exclusive prefix sum of the calling block's VEC_BLOCK values; *total receives their sum
__device__ __forceinline__ int block_exclusive_scan(int x, int *total)
{
    __shared__ int wsum[VEC_BLOCK / 64];
    __shared__ int wtot;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(incl, off);
        if (lane >= off) incl += y;
    }
    __syncthreads();                        // a previous call's readers are done with wsum / wtot
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int k = 0; k < VEC_BLOCK / 64; ++k)
        if (k < w) base += wsum[k];
    if (threadIdx.x == VEC_BLOCK - 1) wtot = base + incl;
    __syncthreads();
    *total = wtot;
    return base + incl - x;
}

// Prefix sums of one or two arrays of the same length in the same launches: out[a][0..n) = exclusive prefix sum
// of in[a][0..n), out[a][n] = the total, also written to total[a] when given.  tsum / toff: per-tile scratch.
struct ScanArgs {
    const int32_t *in[2];
    int32_t *out[2];
    int32_t *tsum[2], *toff[2];
    int32_t *total[2];
    int32_t na;
    int64_t n;
};

__global__ __launch_bounds__(VEC_BLOCK) void scan_tile_sum_kernel(ScanArgs a)
{
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    for (int j = 0; j < a.na; ++j) {
        int s = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k)
            if (b0 + k < a.n) s += a.in[j][b0 + k];
        int tot;
        (void)block_exclusive_scan(s, &tot);
        if (threadIdx.x == 0) a.tsum[j][blockIdx.x] = tot;
    }
}

// one block: out[0..n) = exclusive prefix sum of in[0..n), out[n] = the total (also to *t1 / *t2 when given)
__device__ __forceinline__ void scan_by_one_block(const int32_t *in, int64_t n, int32_t *out, int32_t *t1, int32_t *t2)
{
    int carry = 0;
    for (int64_t t0 = 0; t0 < n; t0 += SCAN_TILE) {
        const int64_t b0 = t0 + (int64_t)threadIdx.x * SCAN_ITEMS;
        int v[SCAN_ITEMS];
        int s = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            v[k] = (b0 + k < n) ? in[b0 + k] : 0;
            s += v[k];
        }
        int tot;
        int run = carry + block_exclusive_scan(s, &tot);
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            if (b0 + k < n) out[b0 + k] = run;
            run += v[k];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        out[n] = carry;
        if (t1) *t1 = carry;
        if (t2) *t2 = carry;
    }
}
// the arrays themselves (short ones)
__global__ __launch_bounds__(VEC_BLOCK) void scan_one_block_kernel(ScanArgs a)
{
    for (int j = 0; j < a.na; ++j) scan_by_one_block(a.in[j], a.n, a.out[j], a.total[j], nullptr);
}
// the tile sums of long arrays: tile offsets, and the grand total to out[n] and total
__global__ __launch_bounds__(VEC_BLOCK) void scan_tiles_kernel(ScanArgs a, int64_t nt)
{
    for (int j = 0; j < a.na; ++j) scan_by_one_block(a.tsum[j], nt, a.toff[j], a.out[j] ? a.out[j] + a.n : nullptr, a.total[j]);
}

__global__ __launch_bounds__(VEC_BLOCK) void scan_tile_apply_kernel(ScanArgs a)
{
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    for (int j = 0; j < a.na; ++j) {
        int v[SCAN_ITEMS];
        int s = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            v[k] = (b0 + k < a.n) ? a.in[j][b0 + k] : 0;
            s += v[k];
        }
        int tot;
        int run = a.toff[j][blockIdx.x] + block_exclusive_scan(s, &tot);
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            if (b0 + k < a.n) a.out[j][b0 + k] = run;
            run += v[k];
        }
    }
}

// scratch: two areas of at least n / SCAN_TILE + 2 elements per array
static void own_scan(ScanArgs a, int32_t *scratch, int64_t area, hipStream_t st)
{
    if (a.n <= 8 * SCAN_TILE) {
        hipLaunchKernelGGL(scan_one_block_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, a);
        return;
    }
    const int64_t nt = (a.n + SCAN_TILE - 1) / SCAN_TILE;
    for (int j = 0; j < a.na; ++j) {
        a.tsum[j] = scratch + (2 * j) * area;
        a.toff[j] = scratch + (2 * j + 1) * area;
    }
    hipLaunchKernelGGL(scan_tile_sum_kernel, dim3((unsigned)nt), dim3(VEC_BLOCK), 0, st, a);
    hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, a, nt);
    hipLaunchKernelGGL(scan_tile_apply_kernel, dim3((unsigned)nt), dim3(VEC_BLOCK), 0, st, a);
}
static void own_scan1(const int32_t *in, int64_t n, int32_t *out, int32_t *total, int32_t *scratch, int64_t area, hipStream_t st)
{
    ScanArgs a{};
    a.in[0] = in;
    a.out[0] = out;
    a.total[0] = total;
    a.na = 1;
    a.n = n;
    own_scan(a, scratch, area, st);
}

// zeroes the multiplicities and the bitmap of sampled rows, empties the rows' lists of sample positions
__global__ __launch_bounds__(VEC_BLOCK) void samp_fill_kernel(int32_t *cnt, int32_t *head, int64_t n, uint32_t *bitmap, int64_t nwords)
{
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < n; i += (int64_t)gridDim.x * VEC_BLOCK) {
        cnt[i] = 0;
        head[i] = -1;
        if (i < nwords) bitmap[i] = 0u;
    }
}
// cnt[r] = how often row r is sampled; bit r of the bitmap = whether it is; head[r], next[head[r]], .. = its sample
// positions (a list per row, in no particular order); len[s] = entries of the row at sample position s
__global__ __launch_bounds__(VEC_BLOCK) void samp_mark_kernel(const int32_t *S, int64_t nS, const int32_t *rowptr, int32_t *cnt,
                                                               uint32_t *bitmap, int32_t *head, int32_t *next, int32_t *len)
{
    for (int64_t s = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; s < nS; s += (int64_t)gridDim.x * VEC_BLOCK) {
        const int32_t r = S[s];
        atomicAdd(&cnt[r], 1);
        atomicOr(&bitmap[r >> 5], 1u << (r & 31));
        next[s] = atomicExch(&head[r], (int32_t)s);
        if (len) len[s] = rowptr[r + 1] - rowptr[r];
    }
}

// The two passes over the whole view's row indices: a thread takes SCAN_ITEMS consecutive entries (two 16-byte
// loads) and asks the bitmap of sampled rows -- copied to LDS when it fits (lds_words > 0), a few KB for tens of
// thousands of rows -- about each; only for the sampled ones does it go on to the multiplicity.
struct SampScan {
    const int32_t *frow;
    int64_t fnnz;
    const uint32_t *bitmap;
    int32_t lds_words;
    const int32_t *cnt;
};
__device__ __forceinline__ void samp_tile_rows(const SampScan &q, const uint32_t *bm_lds, int64_t b0, int (&r)[SCAN_ITEMS],
                                               int (&m)[SCAN_ITEMS])
{
    if (b0 + SCAN_ITEMS <= q.fnnz) {
        const int4 lo = *(const int4 *)(q.frow + b0), hi = *(const int4 *)(q.frow + b0 + 4);
        r[0] = lo.x, r[1] = lo.y, r[2] = lo.z, r[3] = lo.w, r[4] = hi.x, r[5] = hi.y, r[6] = hi.z, r[7] = hi.w;
    } else {
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) r[k] = (b0 + k < q.fnnz) ? q.frow[b0 + k] : -1;
    }
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        m[k] = 0;
        if (r[k] >= 0) {
            const uint32_t w = q.lds_words ? bm_lds[r[k] >> 5] : q.bitmap[r[k] >> 5];
            if ((w >> (r[k] & 31)) & 1u) m[k] = q.cnt[r[k]];
        }
    }
}
__device__ __forceinline__ const uint32_t *samp_bitmap_to_lds(const SampScan &q, uint32_t *lds)
{
    for (int i = threadIdx.x; i < q.lds_words; i += VEC_BLOCK) lds[i] = q.bitmap[i];
    __syncthreads();
    return lds;
}
// tsum[tile] = number of sample entries that the tile's entries of the whole view produce
__global__ __launch_bounds__(VEC_BLOCK) void samp_tile_count_kernel(SampScan q, int32_t *tsum)
{
    static_assert(SCAN_ITEMS == 8, "two 16-byte loads per thread");
    extern __shared__ uint32_t samp_lds[];
    const uint32_t *bm = samp_bitmap_to_lds(q, samp_lds);
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int r[SCAN_ITEMS], m[SCAN_ITEMS];
    samp_tile_rows(q, bm, b0, r, m);
    int s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) s += m[k];
    int tot;
    (void)block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) tsum[blockIdx.x] = tot;
}
// copies the sampled entries of the tile to their places (cap: capacity of the output arrays, never exceeded).
// With `off` (support): also the entry's place in the row-ordered list of the sample's entries, eidx, from its
// place in the CSR arrays (fpos), and its value there (val_in).  The loads of a thread's sampled entries are issued
// together, level by level (entry, first sample position, that position's row pointer): one after the other they
// were a chain of two dozen trips to memory per thread.
// Of the whole view only the places in the CSR arrays (fpos) are read for the sampled entries; column and value
// come from the CSR arrays themselves, where a sampled row's entries are neighbours (a few MB that stay in L2),
// while the view's own column and value arrays would be read at one entry in twenty, i.e. nearly every line of them.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void samp_copy_kernel(SampScan q, const int32_t *colidx, const T *vals, const int32_t *fpos,
                                                              const int32_t *head, const int32_t *next, const int32_t *toff,
                                                              int64_t cap, int32_t *key, int32_t *row, T *val,
                                                              const int32_t *rowptr, const int32_t *off, int32_t *eidx, T *val_in)
{
    extern __shared__ uint32_t samp_lds[];
    const int64_t tile_off = toff[blockIdx.x];
    const uint32_t *bm = samp_bitmap_to_lds(q, samp_lds);
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int r[SCAN_ITEMS], m[SCAN_ITEMS];
    if (b0 + SCAN_ITEMS <= q.fnnz) {
        const int4 lo = *(const int4 *)(q.frow + b0), hi = *(const int4 *)(q.frow + b0 + 4);
        r[0] = lo.x, r[1] = lo.y, r[2] = lo.z, r[3] = lo.w, r[4] = hi.x, r[5] = hi.y, r[6] = hi.z, r[7] = hi.w;
    } else {
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) r[k] = (b0 + k < q.fnnz) ? q.frow[b0 + k] : -1;
    }
    // everything that depends on the row alone is asked for in one go: the multiplicity, the entry's place in the
    // CSR arrays, the row's first sample position, its row pointer
    int32_t col[SCAN_ITEMS], sp[SCAN_ITEMS], within[SCAN_ITEMS], ob[SCAN_ITEMS], rp[SCAN_ITEMS];
    T x[SCAN_ITEMS];
    int s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        m[k] = 0, col[k] = 0, sp[k] = 0, within[k] = 0, ob[k] = 0, rp[k] = 0, x[k] = T(0);
        if (r[k] >= 0) {
            const uint32_t w = q.lds_words ? bm[r[k] >> 5] : q.bitmap[r[k] >> 5];
            if ((w >> (r[k] & 31)) & 1u) {
                m[k] = q.cnt[r[k]];
                within[k] = fpos[b0 + k];                // place in the CSR arrays, for now
                sp[k] = head[r[k]];
                if (off) rp[k] = rowptr[r[k]];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) s += m[k];
    int tot;
    int64_t o = tile_off + block_exclusive_scan(s, &tot);
    if (s == 0) return;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (m[k]) {
            col[k] = colidx[within[k]];
            x[k] = vals[within[k]];
            if (off) {
                within[k] -= rp[k];                      // place of the entry in its row
                ob[k] = off[sp[k]];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (m[k] == 0) continue;
        int32_t spj = sp[k], obj = ob[k];
        for (int j = 0; j < m[k]; ++j, ++o) {
            if (j > 0) {                                 // a row sampled more than once: its next sample position
                spj = next[spj];
                if (off) obj = off[spj];
            }
            if (o >= cap) continue;
            key[o] = col[k];
            row[o] = spj;
            val[o] = x[k];
            if (off) {
                const int64_t e = (int64_t)obj + within[k];
                if (e < cap) {
                    eidx[o] = (int32_t)e;
                    val_in[e] = x[k];
                } else {
                    eidx[o] = 0;
                }
            }
        }
    }
}

// Pieces and distinct columns of the copied list (bound >= *nnz entries): a piece starts at the first entry of a
// column and at every PIECE_LEN-th entry, a column at its first entry.  Both flags are formed from the columns on
// the fly, counted per tile here ...
__device__ __forceinline__ void samp_tile_flags(const int32_t *key, int64_t nnz, int64_t b0, int (&kk)[SCAN_ITEMS],
                                                bool (&pf)[SCAN_ITEMS], bool (&hf)[SCAN_ITEMS])
{
    int prev = (b0 > 0 && b0 - 1 < nnz) ? key[b0 - 1] : -1;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const int64_t t = b0 + k;
        const bool in = t < nnz;
        kk[k] = in ? key[t] : -1;
        hf[k] = in && (t == 0 || kk[k] != prev);
        pf[k] = hf[k] || (in && (t % PIECE_LEN) == 0);
        prev = kk[k];
    }
}
__global__ __launch_bounds__(VEC_BLOCK) void samp_piece_count_kernel(const int32_t *key, const int32_t *nnz_dev, int32_t *tsum_p,
                                                                      int32_t *tsum_h)
{
    const int64_t nnz = *nnz_dev;
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int kk[SCAN_ITEMS];
    bool pf[SCAN_ITEMS], hf[SCAN_ITEMS];
    samp_tile_flags(key, nnz, b0, kk, pf, hf);
    int sp = 0, sh = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) sp += pf[k], sh += hf[k];
    int tp, th;
    (void)block_exclusive_scan(sp, &tp);
    (void)block_exclusive_scan(sh, &th);
    if (threadIdx.x == 0) {
        tsum_p[blockIdx.x] = tp;
        tsum_h[blockIdx.x] = th;
    }
}
// ... and numbered here: piece_start / piece_col of every piece (and the sentinels behind the last), and with
// `support` the distinct columns cols[], the pieces' places among them piece_cpos[], and every entry's place among
// them written at the entry's place in row order: ccol[eidx[t]]
__global__ __launch_bounds__(VEC_BLOCK) void samp_piece_write_kernel(const int32_t *key, const int32_t *nnz_dev, const int32_t *np_dev,
                                                                      const int32_t *toff_p, const int32_t *toff_h, bool support,
                                                                      const int32_t *eidx, int32_t *piece_start, int32_t *piece_col,
                                                                      int32_t *piece_cpos, int32_t *cols, int32_t *ccol)
{
    const int64_t nnz = *nnz_dev;
    const int64_t b0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int kk[SCAN_ITEMS];
    bool pf[SCAN_ITEMS], hf[SCAN_ITEMS];
    samp_tile_flags(key, nnz, b0, kk, pf, hf);
    int sp = 0, sh = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) sp += pf[k], sh += hf[k];
    int tp, th;
    int pid = toff_p[blockIdx.x] + block_exclusive_scan(sp, &tp);
    int rank = toff_h[blockIdx.x] + block_exclusive_scan(sh, &th);
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        const int64_t t = b0 + k;
        if (t < nnz) {
            const int32_t pos = rank + (hf[k] ? 1 : 0) - 1;      // place of the entry's column among the distinct ones
            if (pf[k]) {
                piece_start[pid] = (int32_t)t;
                piece_col[pid] = kk[k];
                if (support) piece_cpos[pid] = pos;
            }
            if (support) {
                if (hf[k]) cols[pos] = kk[k];
                ccol[eidx[t]] = pos;
            }
        }
        pid += pf[k] ? 1 : 0;
        rank += hf[k] ? 1 : 0;
    }
    if (blockIdx.x == 0 && threadIdx.x < 4) {          // the sentinels behind the last piece
        const int32_t np = *np_dev;
        if (threadIdx.x == 0) piece_start[np] = (int32_t)nnz;
        piece_col[np + threadIdx.x] = -1;
        if (support) piece_cpos[np + threadIdx.x] = -1;
    }
}

__global__ __launch_bounds__(VEC_BLOCK) void csr_max_len_kernel(const int32_t *rowptr, int64_t n, int32_t *out)
{
    int m = 0;
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < n; i += (int64_t)gridDim.x * VEC_BLOCK)
        m = max(m, rowptr[i + 1] - rowptr[i]);
    for (int off = 32; off > 0; off >>= 1) m = max(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) atomicMax(out, m);
}

hipError_t csr_max_row_len(const int32_t *rowptr, int64_t n, int32_t *scratch_dev, int32_t *out, hipStream_t st)
{
    CSC_HIP(hipMemsetAsync(scratch_dev, 0, sizeof(int32_t), st));
    if (n > 0) hipLaunchKernelGGL(csr_max_len_kernel, dim3(grid_for(n)), dim3(VEC_BLOCK), 0, st, rowptr, n, scratch_dev);
    CSC_HIP(hipMemcpyAsync(out, scratch_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    return hipStreamSynchronize(st);
}

// The view of rows S[0..nS) (with repeats) as a filter of `full`, the view of all rows of the same matrix, which
// must have kept its entries' places in the CSR arrays (csr_pos).  max_len: the longest row of the matrix
// (nS * max_len bounds the sample's entries and sizes the buffers, so that nothing is allocated here once a
// sample of this many rows has been seen).  One wait for the stream, at the end, for the three counts.  Returns
// hipErrorNotSupported when the bound is too loose to be worth it (more than eight times the average); the
// caller then sorts (csc_build).
hipError_t csc_build_filtered(CscView *v, const CscView &full, int dtype, const int32_t *rowptr, const int32_t *colidx,
                              const void *vals, const int32_t *S, int64_t nS, int64_t n, int32_t max_len, int K,
                              hipStream_t st, bool support)
{
    const size_t es = dtype == SSN_F32 ? 4 : 8;
    v->nnz = 0;
    v->npieces = 0;
    v->win_npieces = -1;                 // the window index of an earlier build is void
    v->ncols = 0;
    v->has_support = false;
    v->nrows = nS;
    const int64_t bound = nS * (int64_t)max_len;
    if (bound == 0 || full.nnz == 0) {
        if (support) {                       // every selected row is empty: row pointers all zero
            CSC_HIP(grow((void **)&v->off, &v->cap_off, nS + 1, sizeof(int32_t)));
            CSC_HIP(hipMemsetAsync(v->off, 0, (size_t)(nS + 1) * sizeof(int32_t), st));
        }
        v->has_support = support;
        return hipSuccess;
    }
    if (!full.csr_pos) return hipErrorNotSupported;
    if (bound >= ((int64_t)1 << 31) - 8 || bound > 8 * (full.nnz / (n > 0 ? n : 1) + 1) * nS) return hipErrorNotSupported;
    if (!v->count_dev) CSC_HIP(hipMalloc((void **)&v->count_dev, 4 * sizeof(int32_t)));
    const int64_t ftiles = (full.nnz + SCAN_TILE - 1) / SCAN_TILE;
    int64_t area = ftiles;                                            // tiles of the longest array scanned here
    if ((bound + SCAN_TILE - 1) / SCAN_TILE > area) area = (bound + SCAN_TILE - 1) / SCAN_TILE;
    if ((n + SCAN_TILE - 1) / SCAN_TILE > area) area = (n + SCAN_TILE - 1) / SCAN_TILE;
    area += 2;
    const int64_t nwords = (n + 31) / 32;
    CSC_HIP(grow((void **)&v->cnt, &v->cap_cnt, n, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->head, &v->cap_head, n, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->bitmap, &v->cap_bitmap, nwords, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->next, &v->cap_next, nS, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->tsum, &v->cap_tsum, ftiles + 2, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->toff, &v->cap_toff, 4 * area, sizeof(int32_t)));        // four scratch areas of the prefix sums
    CSC_HIP(grow((void **)&v->ftoff, &v->cap_ftoff, ftiles + 2, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->key, &v->cap, bound, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->row, &v->cap_row, bound, sizeof(int32_t)));
    CSC_HIP(grow(&v->val, &v->cap_val, bound, es));
    CSC_HIP(grow((void **)&v->piece_start, &v->cap_piece, bound + 1, sizeof(int32_t)));
    CSC_HIP(grow((void **)&v->piece_col, &v->cap_pcol, bound + 4, sizeof(int32_t)));
    // every piece may leave a partial sum and every run of pieces another
    CSC_HIP(grow(&v->piece_part, &v->cap_part, bound * K * 2, es));
    if (support) {
        CSC_HIP(grow((void **)&v->off, &v->cap_off, nS + 1, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->len, &v->cap_len, nS + 1, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->eidx, &v->cap_eidx, bound, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->cols, &v->cap_cols, bound, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->ccol, &v->cap_ccol, bound, sizeof(int32_t)));
        CSC_HIP(grow(&v->val_in, &v->cap_valin, bound, es));
        CSC_HIP(grow((void **)&v->piece_cpos, &v->cap_pcpos, bound + 4, sizeof(int32_t)));
    }
    int32_t *nnz_dev = v->count_dev, *np_dev = v->count_dev + 1, *nc_dev = v->count_dev + 2;

    // 1. how often each row is sampled and at which sample positions; the row pointers of the sample's own CSR form
    hipLaunchKernelGGL(samp_fill_kernel, dim3(grid_for(n)), dim3(VEC_BLOCK), 0, st, v->cnt, v->head, n, (uint32_t *)v->bitmap, nwords);
    hipLaunchKernelGGL(samp_mark_kernel, dim3(grid_for(nS)), dim3(VEC_BLOCK), 0, st, S, nS, rowptr, v->cnt, (uint32_t *)v->bitmap,
                       v->head, v->next, support ? v->len : nullptr);
    if (support) own_scan1(v->len, nS, v->off, nullptr, v->toff, area, st);
    // 2. count per tile of the whole view, places of the tiles, copy
    SampScan q{};
    q.frow = full.row;
    q.fnnz = full.nnz;
    q.bitmap = (const uint32_t *)v->bitmap;
    q.lds_words = nwords <= 12288 ? (int32_t)nwords : 0;          // up to 48 KB of LDS
    q.cnt = v->cnt;
    const size_t lds = (size_t)q.lds_words * sizeof(uint32_t);
    hipLaunchKernelGGL(samp_tile_count_kernel, dim3((unsigned)ftiles), dim3(VEC_BLOCK), lds, st, q, v->tsum);
    own_scan1(v->tsum, ftiles, v->ftoff, nnz_dev, v->toff, area, st);
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(samp_copy_kernel<float>, dim3((unsigned)ftiles), dim3(VEC_BLOCK), lds, st, q, colidx,
                           (const float *)vals, full.csr_pos, v->head, v->next, v->ftoff, bound, v->key, v->row,
                           (float *)v->val, rowptr, support ? v->off : nullptr, v->eidx, (float *)v->val_in);
    else
        hipLaunchKernelGGL(samp_copy_kernel<double>, dim3((unsigned)ftiles), dim3(VEC_BLOCK), lds, st, q, colidx,
                           (const double *)vals, full.csr_pos, v->head, v->next, v->ftoff, bound, v->key, v->row,
                           (double *)v->val, rowptr, support ? v->off : nullptr, v->eidx, (double *)v->val_in);
    // 3. pieces, distinct columns: flags counted per tile, the tiles' counts summed up, everything numbered
    {
        const int64_t stiles = (bound + SCAN_TILE - 1) / SCAN_TILE;
        ScanArgs a{};
        a.n = bound;
        a.na = 2;
        for (int j = 0; j < 2; ++j) {
            a.tsum[j] = v->toff + (2 * j) * area;
            a.toff[j] = v->toff + (2 * j + 1) * area;
        }
        a.total[0] = np_dev;
        a.total[1] = nc_dev;
        hipLaunchKernelGGL(samp_piece_count_kernel, dim3((unsigned)stiles), dim3(VEC_BLOCK), 0, st, v->key, nnz_dev, a.tsum[0],
                           a.tsum[1]);
        hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, a, stiles);
        hipLaunchKernelGGL(samp_piece_write_kernel, dim3((unsigned)stiles), dim3(VEC_BLOCK), 0, st, v->key, nnz_dev, np_dev,
                           a.toff[0], a.toff[1], support, v->eidx, v->piece_start, v->piece_col, v->piece_cpos, v->cols, v->ccol);
    }
    CSC_HIP(hipGetLastError());
    int32_t counts[3] = {0, 0, 0};
    CSC_HIP(hipMemcpyAsync(counts, v->count_dev, 3 * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    CSC_HIP(hipStreamSynchronize(st));
    if (counts[0] < 0 || counts[0] > bound) return hipErrorInvalidValue;
    v->nnz = counts[0];
    v->npieces = counts[0] ? counts[1] : 0;
    v->ncols = (support && counts[0]) ? counts[2] : 0;
    v->has_support = support;
    return hipSuccess;
}

// ---- the product ----------------------------------------------------------------------------
struct CscApply {
    const int32_t *row, *piece_start, *piece_col;
    const void *val;
    int32_t npieces;
    int64_t nnz;
    int32_t K, KP;
    const void *U;           // rows indexed by the view's sample positions, stride KP
    void *out;               // p x ldo, receives += coef * X^T U
    int64_t ldo;
    double coef;
    const CgSlot *slot;      // nullable: coef *= -slot->alpha; nothing happens once that CG loop has ended
    void *piece_part;
    void *run_part;          // sums of runs of pieces (grouped combine), laid out like piece_part
    int32_t look;            // pieces a wave of the run / combine kernels looks at (a power of two, 4..64)
    const int32_t *skip;
    const int32_t *key;      // column of every entry (csc1_window_kernel: where the pieces of a window start)
    const int32_t *win_pid;  // piece that starts at entry 64 w (csc1_window_kernel)
};
// (piece_col may be the pieces' columns or their positions among the distinct columns: equal columns have
// equal positions, and the result row written is whichever of the two the caller's `out` is indexed by)

// lane group (slot) g of a wave = K lanes, one per class; NS = 64 / K groups per wave, one piece per group
template <typename T> __global__ __launch_bounds__(256) void csc_piece_kernel(CscApply a)
{
    if (a.skip && *a.skip) return;
    double coef = a.coef;
    if (a.slot) {
        if (a.slot->done || a.slot->brk) return;
        coef *= -a.slot->alpha;
    }
    // no lane leaves before the shuffles below: a lane without a piece (spare lanes of the wave, groups past the
    // last piece) walks through them with an empty piece
    const int lane = threadIdx.x & 63;
    const int K = a.K, NS = 64 / K;
    const int s = lane / K, c = lane - s * K;
    const int64_t pid = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * NS + s;
    const bool active = s < NS && pid < a.npieces;
    const T *val = (const T *)a.val;
    const T *U = (const T *)a.U;
    const int64_t t0 = active ? a.piece_start[pid] : 0, t1 = active ? a.piece_start[pid + 1] : 0;
    const int col = active ? a.piece_col[pid] : 0;
    const bool head = active && ((pid == 0) || (a.piece_col[pid - 1] != col));
    const bool more = active && a.piece_col[pid + 1] == col;
    // the result element this piece adds into (a whole column in one piece) is fetched now: its trip to memory
    // then overlaps the gathers below instead of following them
    T *o = (T *)a.out + (int64_t)col * a.ldo + c;
    const T oval = (head && !more) ? *o : T(0);
    // Entries are fetched K at a time, one per lane of the group (one coalesced load of row positions and one
    // of values instead of K broadcast loads each), and handed round the group by lane shuffles; the gathers
    // of U, four in flight, are then the only loads in the loop.  The groups of a wave have different piece
    // lengths, so the loops run to the longest and the shorter groups add zeros.
    T a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    const int gbase = s * K;
    const int len = (int)(t1 - t0);
    if (K < 4) {
        // Groups this narrow would fetch one to three entries per round of the exchange below, a chain of index ->
        // gather round trips per entry.  Every lane of the group reads the entries itself instead (the same
        // addresses across the group), eight in flight.
        for (int b = 0; b < len; b += 8) {
            int r[8];
            T v[8], u[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool have = b + k < len;
                r[k] = have ? a.row[t0 + b + k] : -1;
                v[k] = have ? val[t0 + b + k] : T(0);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) u[k] = (r[k] >= 0) ? U[(int64_t)r[k] * a.KP + c] : T(0);
            a0 += v[0] * u[0];
            a1 += v[1] * u[1];
            a2 += v[2] * u[2];
            a3 += v[3] * u[3];
            a0 += v[4] * u[4];
            a1 += v[5] * u[5];
            a2 += v[6] * u[6];
            a3 += v[7] * u[7];
        }
        if (!active) return;
        const T accn = (a0 + a1) + (a2 + a3);
        if (head && !more) {
            *o = (T)((double)oval + coef * (double)accn);
        } else {
            ((T *)a.piece_part)[pid * K + c] = accn;
        }
        return;
    }
    // Waves whose pieces all have at most four entries -- most of them, on text-like data, where most columns
    // appear in a handful of the selected rows -- take them without the exchange: every lane of the group reads
    // the (up to four) entries itself, all at once, and the gathers follow.
    if (!__any(len > 4)) {
        int r[4];
        T v[4], u[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool have = k < len;
            r[k] = have ? a.row[t0 + k] : -1;
            v[k] = have ? val[t0 + k] : T(0);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) u[k] = (r[k] >= 0) ? U[(int64_t)r[k] * a.KP + c] : T(0);
        if (!active) return;
        const T accs = (v[0] * u[0] + v[1] * u[1]) + (v[2] * u[2] + v[3] * u[3]);
        if (head && !more) {
            *o = (T)((double)oval + coef * (double)accs);
        } else {
            ((T *)a.piece_part)[pid * K + c] = accs;
        }
        return;
    }
    int maxlen = len;
    for (int off = 32; off > 0; off >>= 1) maxlen = max(maxlen, __shfl_xor(maxlen, off));
    for (int b = 0; b < maxlen; b += K) {
        const int mine = b + c;
        const bool have = mine < len;
        const int rmine = have ? a.row[t0 + mine] : 0;
        const T vmine = have ? val[t0 + mine] : T(0);
        const int nb = min(K, maxlen - b);                       // uniform over the wave
        for (int j = 0; j < nb; j += 4) {
            int r[4];
            T v[4], u[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int src = gbase + ((j + k < K) ? j + k : 0);
                r[k] = __shfl(rmine, src);
                v[k] = __shfl(vmine, src);
                if (j + k >= nb || b + j + k >= len) v[k] = T(0), r[k] = r[0];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) u[k] = U[(int64_t)r[k] * a.KP + c];
            a0 += v[0] * u[0];
            a1 += v[1] * u[1];
            a2 += v[2] * u[2];
            a3 += v[3] * u[3];
        }
    }
    const T acc = (a0 + a1) + (a2 + a3);
    if (!active) return;
    if (head && !more) {
        *o = (T)((double)oval + coef * (double)acc);
    } else {
        ((T *)a.piece_part)[pid * K + c] = acc;
    }
}

// One weight column (the binary problem): the job of csc_piece_kernel with a lane per ENTRY instead of a lane per
// piece.  With K = 1 a lane group is a single lane that walks its piece of up to 64 entries alone, so the lanes of a
// wave read 64 different stretches of the entry arrays; here a wave takes one aligned window of 64 entries (pieces
// start at every 64th entry, so a window holds whole pieces) and reads rows, values and the gathered u coalesced.
// The products are added along the wave by an inclusive scan on the vector units (fp64 in both precisions); then the
// lanes change roles: lane j stands for the window's j-th piece, reads where it starts and ends (coalesced) and takes
// its sum as the difference of the scan values at its last entry and before its first.  The piece's lane adds a
// whole column into the result or leaves the piece's partial sum, exactly as csc_piece_kernel does;
// csc1_combine_kernel then adds the partial sums of the columns of several pieces.
template <typename T> __global__ __launch_bounds__(256) void csc1_window_kernel(CscApply a)
{
    if (a.skip && *a.skip) return;
    double coef = a.coef;
    if (a.slot) {
        if (a.slot->done || a.slot->brk) return;
        coef *= -a.slot->alpha;
    }
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w * 64 >= a.nnz) return;                                 // the whole wave
    const int64_t e = w * 64 + lane;
    const bool have = e < a.nnz;
    const int r = have ? a.row[e] : 0;
    const T v = have ? ((const T *)a.val)[e] : T(0);
    // this lane's piece in its second role: the window's pieces are win_pid[w] .. (next window's first piece) - 1
    const int64_t pid0 = a.win_pid[w];
    const int64_t pend = ((w + 1) * 64 < a.nnz) ? (int64_t)a.win_pid[w + 1] : (int64_t)a.npieces;
    const int64_t pid = pid0 + lane;
    const bool piece = pid < pend;
    const int64_t pq = piece ? pid : pid0;                       // (lanes without a piece read the first one's numbers)
    const int ps = a.piece_start[pq], pe = a.piece_start[pq + 1];
    const int ocol = a.piece_col[pq];
    const int pcol = (pq > 0) ? a.piece_col[pq - 1] : -2;
    const int ncol = a.piece_col[pq + 1];
    const double x = have ? (double)v * (double)((const T *)a.U)[(int64_t)r * a.KP] : 0.0;
    const double P = wave_inclusive_scan(x);
    const int b = ps - (int)(w * 64), en = pe - (int)(w * 64);   // 0 <= b < en <= 64
    const double Pe = __shfl(P, en - 1), Pb = __shfl(P, b > 0 ? b - 1 : 0);
    if (piece) {
        const T sum = (T)((b > 0) ? Pe - Pb : Pe);
        const bool head = ocol != pcol, more = ncol == ocol;
        if (head && !more) {
            T *o = (T *)a.out + (int64_t)ocol * a.ldo;
            *o = (T)((double)*o + coef * (double)sum);
        } else {
            ((T *)a.piece_part)[pid] = sum;
        }
    }
}

// One weight column, second and last kernel: the partial sums of the columns of several pieces, added with a lane per
// PIECE.  A wave takes 64 consecutive pieces and adds, by the same segmented reduction, the pieces of every column
// that starts among them; a column that runs on behind the wave's last piece (only the last one can) is followed by
// the whole wave, 64 pieces per step, until it ends -- a column present in most of 65 000 rows has a thousand pieces,
// which one lane adding them one after the other would be a chain of as many trips to memory.  Fixed orders, one
// writer per column.  (The columns of a single piece were added by csc1_window_kernel.)
template <typename T> __global__ __launch_bounds__(256) void csc1_combine_kernel(CscApply a)
{
    if (a.skip && *a.skip) return;
    double coef = a.coef;
    if (a.slot) {
        if (a.slot->done || a.slot->brk) return;
        coef *= -a.slot->alpha;
    }
    const int lane = threadIdx.x & 63;
    const int64_t base = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 64;
    if (base >= a.npieces) return;                               // the whole wave
    const int64_t pid = base + lane;
    const bool have = pid < a.npieces;
    const T *pp = (const T *)a.piece_part;
    const int col = have ? a.piece_col[pid] : -1;
    const int prevc = (have && pid > 0) ? a.piece_col[pid - 1] : -2;
    const int nextc = have ? a.piece_col[pid + 1] : -3;          // (sentinels -1 behind the last piece)
    const bool head = have && col != prevc, more = have && nextc == col;
    const bool multi = have && !(head && !more);                 // piece of a column of several pieces: it left a partial sum
    T x = multi ? pp[pid] : T(0);
    const int below = __shfl_up(col, 1);                         // (every lane takes part in the exchange)
    const bool start = lane == 0 || col != below;
    const unsigned long long starts = __ballot(start);
    const unsigned long long above = (lane == 63) ? 0ull : ((starts >> (lane + 1)) << (lane + 1));
    const int send = above ? (__ffsll((long long)above) - 2) : 63;
    for (int d = 1; d < 64; d <<= 1) {
        const T y = __shfl_down(x, d);
        if (lane + d <= send) x += y;
    }
    // The column of the wave's last piece may run on behind it; this wave follows it if the column starts here
    // (the wave where it starts does otherwise).
    const int lastcol = __shfl(col, 63);
    const int lastnext = __shfl(nextc, 63);
    const int laststart = 63 - __clzll(starts);                  // first lane of the last segment (lane 0 always starts one)
    const int lasthead = __shfl((int)head, laststart);
    T csum = T(0);
    if (lastcol >= 0 && lastnext == lastcol && lasthead) {       // uniform over the wave
        // 256 pieces per step, all their loads requested together (a piece that is not this column's is read and
        // dropped); the step's sum is the last lane's value of a scan over the lanes
        for (int64_t j0 = base + 64;; j0 += 256) {
            T y[4];
            bool m[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int64_t j = j0 + 64 * k + lane, jc = j < a.npieces ? j : (int64_t)a.npieces - 1;
                const int c = a.piece_col[jc];
                const T pv = pp[jc];
                m[k] = j < a.npieces && c == lastcol;
                y[k] = m[k] ? pv : T(0);
            }
            const double t = ((double)y[0] + (double)y[1]) + ((double)y[2] + (double)y[3]);
            csum += (T)__shfl(wave_inclusive_scan(t), 63);
            if (!__all(m[3])) break;
        }
    }
    if (start && head && more) {                                 // first piece of a column of several: the column's writer
        const T total = (send == 63) ? x + csum : x;
        T *o = (T *)a.out + (int64_t)col * a.ldo;
        *o = (T)((double)*o + coef * (double)total);
    }
}

// win_pid[w] = the piece that starts at entry 64 w (every aligned 64th entry starts one)
__global__ __launch_bounds__(VEC_BLOCK) void csc_window_index_kernel(const int32_t *piece_start, int32_t npieces, int32_t *win_pid)
{
    const int64_t k = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x;
    if (k >= npieces) return;
    const int32_t t = piece_start[k];
    if ((t & 63) == 0) win_pid[t >> 6] = (int32_t)k;
}

hipError_t csc_window_index(CscView *v, hipStream_t st)
{
    const int64_t nwin = (v->nnz + 63) / 64;
    if (nwin > v->cap_win) {
        if (v->win_pid) {
            CSC_HIP(hipStreamSynchronize(st));
            CSC_HIP(hipFree(v->win_pid));
            v->win_pid = nullptr;
        }
        const int64_t cap = nwin + nwin / 4 + 16;
        CSC_HIP(hipMalloc((void **)&v->win_pid, (size_t)cap * sizeof(int32_t)));
        v->cap_win = cap;
    }
    v->win_npieces = v->npieces;
    if (v->npieces > 0)
        hipLaunchKernelGGL(csc_window_index_kernel, dim3((unsigned)((v->npieces + VEC_BLOCK - 1) / VEC_BLOCK)), dim3(VEC_BLOCK), 0, st,
                           v->piece_start, v->npieces, v->win_pid);
    return hipGetLastError();
}

// Columns of several pieces: a lane group adds the column's partial sums in piece order and adds the result into
// the output.  Most pieces are whole columns with nothing to combine, so a wave first looks at up to 64 pieces, one
// per lane, and its lane groups then take the pieces that have work, NS at a time (a group per piece from the start
// was twenty times the waves, nearly all of which looked at three numbers and left).
// GROUPED: the pieces of a column are first added in runs that end at every CSC_RUN-th piece (csc_run_kernel, any
// number of runs at a time), and the first piece's group adds the runs: a column present in most of 20 000 rows has
// some 300 pieces, and adding them one after the other is a chain of 80 round trips to memory.
constexpr int CSC_RUN = 16;

// the lane (0..63) whose piece group s of the wave takes next, or -1; *mask loses the NS lowest set bits
__device__ __forceinline__ int csc_take(unsigned long long *mask, int s, int NS)
{
    unsigned long long m = *mask;
    int mine = -1;
    for (int i = 0; i < NS && m; ++i) {
        if (i == s) mine = __ffsll((long long)m) - 1;
        m &= m - 1;
    }
    *mask = m;
    return mine;
}

template <typename T> __global__ __launch_bounds__(256) void csc_run_kernel(CscApply a)
{
    if (a.skip && *a.skip) return;
    if (a.slot && (a.slot->done || a.slot->brk)) return;
    const int lane = threadIdx.x & 63;
    const int K = a.K, NS = 64 / K;
    const int s = lane / K, c = lane - s * K;
    const int64_t base = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * a.look;
    bool starts = false;                       // a run starts at a column's first piece and at every CSC_RUN-th
    {                                          // piece; whole columns have none
        const int64_t pid = base + lane;
        if (lane < a.look && pid < a.npieces) {
            const int col = a.piece_col[pid];
            const bool head = (pid == 0) || (a.piece_col[pid - 1] != col);
            starts = head ? (a.piece_col[pid + 1] == col) : (pid % CSC_RUN == 0);
        }
    }
    unsigned long long mask = __ballot(starts);
    const T *pp = (const T *)a.piece_part;
    while (mask) {
        const int mine = csc_take(&mask, s, NS);
        if (s >= NS || mine < 0) continue;
        const int64_t pid = base + mine;
        const int col = a.piece_col[pid];
        T acc = pp[pid * K + c];
        for (int64_t j = pid + 1; j % CSC_RUN != 0; j += 4) {      // four pieces per round; the adds keep the order
            const bool m0 = a.piece_col[j] == col, m1 = m0 && (j + 1) % CSC_RUN != 0 && a.piece_col[j + 1] == col;
            const bool m2 = m1 && (j + 2) % CSC_RUN != 0 && a.piece_col[j + 2] == col;
            const bool m3 = m2 && (j + 3) % CSC_RUN != 0 && a.piece_col[j + 3] == col;
            const T p0 = m0 ? pp[j * K + c] : T(0), p1 = m1 ? pp[(j + 1) * K + c] : T(0);
            const T p2 = m2 ? pp[(j + 2) * K + c] : T(0), p3 = m3 ? pp[(j + 3) * K + c] : T(0);
            acc += p0;
            acc += p1;
            acc += p2;
            acc += p3;
            if (!m3 || (j + 4) % CSC_RUN == 0) break;
        }
        ((T *)a.run_part)[pid * K + c] = acc;
    }
}

template <typename T, bool GROUPED> __global__ __launch_bounds__(256) void csc_combine_kernel(CscApply a)
{
    if (a.skip && *a.skip) return;
    double coef = a.coef;
    if (a.slot) {
        if (a.slot->done || a.slot->brk) return;
        coef *= -a.slot->alpha;
    }
    const int lane = threadIdx.x & 63;
    const int K = a.K, NS = 64 / K;
    const int s = lane / K, c = lane - s * K;
    const int64_t base = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * a.look;
    bool first = false;                        // first piece of a column of several
    {
        const int64_t pid = base + lane;
        if (lane < a.look && pid < a.npieces) {
            const int col = a.piece_col[pid];
            const bool head = (pid == 0) || (a.piece_col[pid - 1] != col);
            first = head && a.piece_col[pid + 1] == col;
        }
    }
    unsigned long long mask = __ballot(first);
    while (mask) {
        const int mine = csc_take(&mask, s, NS);
        if (s >= NS || mine < 0) continue;
        const int64_t pid = base + mine;
        const int col = a.piece_col[pid];
        T *o = (T *)a.out + (int64_t)col * a.ldo + c;
        const T oval = *o;                       // fetched before the partial sums, not after them
        T acc;
        if constexpr (GROUPED) {
            const T *rp = (const T *)a.run_part;
            acc = rp[pid * K + c];
            const int64_t np = a.npieces;
            for (int64_t j = (pid / CSC_RUN + 1) * CSC_RUN;; j += 4 * CSC_RUN) {     // four runs per round, in order
                const int64_t j1 = j + CSC_RUN, j2 = j + 2 * CSC_RUN, j3 = j + 3 * CSC_RUN;
                const bool m0 = j < np && a.piece_col[j] == col, m1 = m0 && j1 < np && a.piece_col[j1] == col;
                const bool m2 = m1 && j2 < np && a.piece_col[j2] == col, m3 = m2 && j3 < np && a.piece_col[j3] == col;
                const T p0 = m0 ? rp[j * K + c] : T(0), p1 = m1 ? rp[j1 * K + c] : T(0);
                const T p2 = m2 ? rp[j2 * K + c] : T(0), p3 = m3 ? rp[j3 * K + c] : T(0);
                acc += p0;
                acc += p1;
                acc += p2;
                acc += p3;
                if (!m3) break;
            }
        } else {
            const T *pp = (const T *)a.piece_part;
            acc = pp[pid * K + c];
            for (int64_t j = pid + 1;; j += 4) {     // four pieces per round; the adds keep the piece order
                const bool m0 = a.piece_col[j] == col, m1 = m0 && a.piece_col[j + 1] == col;
                const bool m2 = m1 && a.piece_col[j + 2] == col, m3 = m2 && a.piece_col[j + 3] == col;
                const T p0 = m0 ? pp[j * K + c] : T(0), p1 = m1 ? pp[(j + 1) * K + c] : T(0);
                const T p2 = m2 ? pp[(j + 2) * K + c] : T(0), p3 = m3 ? pp[(j + 3) * K + c] : T(0);
                acc += p0;
                acc += p1;
                acc += p2;
                acc += p3;
                if (!m3) break;
            }
        }
        *o = (T)((double)oval + coef * (double)acc);
    }
}

// out += coef * X_view^T U  (out already holds whatever the product is added to: lambda * M, or the CG
// residual).  K <= 64.
hipError_t launch_csc_apply(int dtype, const CscView &v, int K, int KP, const void *U, double coef, void *out, int64_t ldo,
                            const CgSlot *slot, const int32_t *skip, hipStream_t st, bool support_coords)
{
    if (v.npieces == 0) return hipSuccess;
    if (support_coords && !v.has_support) return hipErrorInvalidValue;
    CscApply a{};
    a.row = v.row;
    a.piece_start = v.piece_start;
    a.piece_col = support_coords ? v.piece_cpos : v.piece_col;
    a.val = v.val;
    a.npieces = v.npieces;
    a.nnz = v.nnz;
    a.K = K;
    a.KP = KP;
    a.U = U;
    a.out = out;
    a.ldo = ldo;
    a.coef = coef;
    a.slot = slot;
    a.piece_part = v.piece_part;
    const size_t es = dtype == SSN_F32 ? 4 : 8;
    a.run_part = (char *)v.piece_part + (size_t)v.npieces * K * es;
    a.skip = skip;
    a.key = v.key;
    a.win_pid = v.win_pid;
    // one weight column: a lane per entry (csc1_window_kernel) where the view carries its window index
    const bool windows = K == 1 && v.win_pid && v.win_npieces == v.npieces && v.key;
    const unsigned wblocks = (unsigned)((((v.nnz + 63) / 64) + 3) / 4);
    const unsigned pblocks = (unsigned)(((((int64_t)v.npieces + 63) / 64) + 3) / 4);
    const int NS = 64 / K;
    const int64_t waves = ((int64_t)v.npieces + NS - 1) / NS;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    // a column has at most one entry per selected row: views of few rows have short columns everywhere, and the
    // run kernel would only add a launch to each of their products
    const bool grouped = v.nrows > (int64_t)PIECE_LEN * 2 * CSC_RUN;
    // a wave of the run / combine kernels looks at `look` pieces: 64 on large views; fewer on small ones, whose
    // pieces with work would otherwise queue up in too few waves
    int look = 64;
    while (look > 4 && (int64_t)v.npieces / look < 8192) look >>= 1;
    a.look = look;
    const unsigned cblocks = (unsigned)((((int64_t)v.npieces + look - 1) / look + 3) / 4);
    if (dtype == SSN_F32) {
        if (windows) {
            hipLaunchKernelGGL(csc1_window_kernel<float>, dim3(wblocks), dim3(256), 0, st, a);
            hipLaunchKernelGGL(csc1_combine_kernel<float>, dim3(pblocks), dim3(256), 0, st, a);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(csc_piece_kernel<float>, dim3(blocks), dim3(256), 0, st, a);
        if (grouped) {
            hipLaunchKernelGGL(csc_run_kernel<float>, dim3(cblocks), dim3(256), 0, st, a);
            hipLaunchKernelGGL((csc_combine_kernel<float, true>), dim3(cblocks), dim3(256), 0, st, a);
        } else {
            hipLaunchKernelGGL((csc_combine_kernel<float, false>), dim3(cblocks), dim3(256), 0, st, a);
        }
    } else {
        if (windows) {
            hipLaunchKernelGGL(csc1_window_kernel<double>, dim3(wblocks), dim3(256), 0, st, a);
            hipLaunchKernelGGL(csc1_combine_kernel<double>, dim3(pblocks), dim3(256), 0, st, a);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(csc_piece_kernel<double>, dim3(blocks), dim3(256), 0, st, a);
        if (grouped) {
            hipLaunchKernelGGL(csc_run_kernel<double>, dim3(cblocks), dim3(256), 0, st, a);
            hipLaunchKernelGGL((csc_combine_kernel<double, true>), dim3(cblocks), dim3(256), 0, st, a);
        } else {
            hipLaunchKernelGGL((csc_combine_kernel<double, false>), dim3(cblocks), dim3(256), 0, st, a);
        }
    }
    return hipGetLastError();
}

}  // namespace ssn
