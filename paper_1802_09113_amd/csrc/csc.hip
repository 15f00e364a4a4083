// Column-sorted view of a set of CSR rows and the transposed product X_rows^T U on it.
//
// The transposed product of eq. (13) / Alg. 6 adds x_ij * u_i into row j of the result for every stored
// entry.  Scattering from the CSR rows would need floating-point atomics (an order of summation that
// changes from run to run); instead the entries of the selected rows are sorted by column once -- when
// the context first needs the whole matrix, and at every ssn_hess_prepare for the sample -- and each
// product then GATHERS: the entries of a column are consecutive, rows of U are read, and every result
// element has exactly one writer and one order of summation.
//
// Work is cut into pieces: a piece ends where the column changes and at every PIECE_LEN-th entry, so hot
// columns (a few appear in almost every row of text-like data) are spread over many lane groups.  A
// piece that is a whole column adds into the result directly; the pieces of a longer column leave
// partial sums that a second kernel adds in piece order.
//
// The one-off construction uses hipCUB's device radix sort and prefix sums; the product kernels are
// hand-written.
#include "ssn_internal.h"

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
                   v->row_in, v->val_in, v->flag, v->pid, v->cub_tmp, v->count_dev, v->cols, v->ccol, v->piece_cpos};
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
    v->cap_in = v->cap_flag = v->cap_pid = 0;
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
    v->ncols = 0;
    v->has_support = false;
    if (!v->count_dev) CSC_HIP(hipMalloc((void **)&v->count_dev, 2 * sizeof(int32_t)));

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
        int64_t c0 = v->cap_in, c1 = v->cap_in, c2 = v->cap_in, c3 = v->cap_in, c4 = v->cap_in;
        CSC_HIP(grow((void **)&v->key_in, &c0, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->idx_in, &c1, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->idx_out, &c2, nnz, sizeof(int32_t)));
        CSC_HIP(grow((void **)&v->row_in, &c3, nnz, sizeof(int32_t)));
        CSC_HIP(grow(&v->val_in, &c4, nnz, es));
        v->cap_in = c0;
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
        hipLaunchKernelGGL(csc_piece_kernel<float>, dim3(blocks), dim3(256), 0, st, a);
        if (grouped) {
            hipLaunchKernelGGL(csc_run_kernel<float>, dim3(cblocks), dim3(256), 0, st, a);
            hipLaunchKernelGGL((csc_combine_kernel<float, true>), dim3(cblocks), dim3(256), 0, st, a);
        } else {
            hipLaunchKernelGGL((csc_combine_kernel<float, false>), dim3(cblocks), dim3(256), 0, st, a);
        }
    } else {
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
