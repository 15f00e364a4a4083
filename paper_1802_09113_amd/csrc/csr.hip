// CSR kernels: row-per-wavefront SpMM with the per-row epilogue fused in (the transposed product is in
// csc.hip).
//
// rows kernel: one wavefront owns one row at a time.  Lanes are split as (slot, class): NS = 64/K
// stored entries are processed per step, lane (s,c) gathers M[col_s, c] -- the K values of one feature
// are contiguous (feature-major weights), so one stored entry fetches one contiguous K-vector.
#include "ssn_internal.h"
#include "ssn_math.h"

#include <limits>

namespace ssn {

__device__ __forceinline__ float c_exp(float x) { return expf(x); }
__device__ __forceinline__ double c_exp(double x) { return exp_nonpos(x, opaque_zero()); }      // arguments are <= 0 here
__device__ __forceinline__ float c_log(float x) { return logf(x); }
__device__ __forceinline__ double c_log(double x) { return log_ge1(x, opaque_zero()); }           // alpha >= 1

template <typename T> __device__ __forceinline__ T wave_sum(T x)
{
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}
template <typename T> __device__ __forceinline__ T wave_max(T x)
{
    for (int off = 32; off > 0; off >>= 1) x = fmax(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ int wave_min_int(int x)
{
    for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off));
    return x;
}

// z_c = sum over the row's stored entries of x * M[col, c]; result valid in lanes c < K.
// (b, e: the row's range of stored entries, loaded by the caller one row ahead)
template <typename T>
__device__ __forceinline__ T csr_row_margin(const RowsArgs &a, int64_t b, int64_t e, int lane, int K, int NS)
{
    const int s = lane / K, c = lane - s * K;
    const bool act = s < NS;
    const T *vals = (const T *)a.vals;
    const T *M = (const T *)a.M;
    // eight stored entries per lane in flight: a row's gathers depend on its column indices, and a single chain
    // of index -> gather round trips is what bounds a wave that owns a whole row (four in flight: the sampled
    // product's rows kernel took 26 us instead of 21 on the sparse workload, the fp32 objective 150 instead of 136)
    T acc = 0;
    if (act) {
        constexpr int U = 8;
        T av[U];
#pragma unroll
        for (int u = 0; u < U; ++u) av[u] = 0;
        int64_t t = b + s;
        for (; t + (U - 1) * NS < e; t += U * NS) {
            int64_t cc[U];
            T vv[U], mm[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cc[u] = a.colidx[t + u * NS];
#pragma unroll
            for (int u = 0; u < U; ++u) vv[u] = vals[t + u * NS];
#pragma unroll
            for (int u = 0; u < U; ++u) mm[u] = M[cc[u] * a.ldm + c];
#pragma unroll
            for (int u = 0; u < U; ++u) av[u] += vv[u] * mm[u];
        }
        if (t + NS < e) {          // two or more entries left for this lane: the same round with lanes switched off
            int64_t cc[U];
            T vv[U], mm[U];
#pragma unroll
            for (int u = 0; u < U; ++u) cc[u] = (t + u * NS < e) ? (int64_t)a.colidx[t + u * NS] : (int64_t)-1;
#pragma unroll
            for (int u = 0; u < U; ++u) vv[u] = (t + u * NS < e) ? vals[t + u * NS] : T(0);
#pragma unroll
            for (int u = 0; u < U; ++u) mm[u] = (cc[u] >= 0) ? M[cc[u] * a.ldm + c] : T(0);
#pragma unroll
            for (int u = 0; u < U; ++u) av[u] += vv[u] * mm[u];
        } else if (t < e) {
            av[0] += vals[t] * M[(int64_t)a.colidx[t] * a.ldm + c];
        }
#pragma unroll
        for (int u = 1; u < U; ++u) av[0] += av[u];
        acc = av[0];
    }
    // fold the NS slots onto slot 0: a tree over the slots (log2 NS steps in a fixed order; with one weight column a
    // wave holds 64 slots, and adding them one after the other was most of a short row's time)
    int top = 1;
    while (top < NS) top <<= 1;
    T tot = acc;
    for (int h = top >> 1; h >= 1; h >>= 1) {
        const T o = __shfl(tot, (lane + h * K) & 63);
        if (s + h < NS) tot += o;
    }
    return (lane < K) ? tot : T(0);
}

// SPLIT: a pass over few, long rows (the sampled rows of a matrix with hundreds of entries per row) leaves most of
// the chip idle with a wave per row, and each wave with a long chain of rounds.  There a WORKGROUP owns a row: its
// four waves take a quarter of the row's entries each (whole rounds of NS entries), leave their partial margins in
// LDS, and every wave adds the four in the same order; wave 0 does the row's stores and sums.  All waves of a
// workgroup walk the same rows, so the barrier is reached by all; the partials alternate between two buffers, so one
// barrier per row is enough.
template <typename T, int MODE, bool SPLIT = false>
__global__ __launch_bounds__(64 * ROWS_WAVES_PER_BLOCK) void csr_rows_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const int64_t nwaves = SPLIT ? (int64_t)gridDim.x : (int64_t)gridDim.x * ROWS_WAVES_PER_BLOCK;    // stride over the rows
    const int64_t wave = (int64_t)blockIdx.x * ROWS_WAVES_PER_BLOCK + wib;
    const int K = a.K;
    const int NS = 64 / K;
    const bool cv = lane < K && (!SPLIT || wib == 0);            // lanes that hold (and store) a row's K values
    __shared__ T zs[SPLIT ? 2 * ROWS_WAVES_PER_BLOCK * 64 : 1];
    int par = 0;
    const T NEG = -std::numeric_limits<T>::infinity();
    double loss = 0.0;
    int hits = 0;

    // A wave's rows are chains of dependent trips to memory (row pointers -> entries -> rows of M -> label): the
    // pointers and the label of the NEXT row are requested before the current row's work, so that only the entries
    // and the gathers of a row wait for each other.
    int64_t sv = SPLIT ? (int64_t)blockIdx.x : wave, svn = 0, row = 0, rown = 0, b = 0, e = 0, bn = 0, en = 0;
    int lab = 0, labn = 0;
    constexpr bool NEED_LAB = (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_PRED);
    if (sv < a.nrows) {
        row = a.S ? a.S[sv] : sv;
        b = a.rowptr[row];
        e = a.rowptr[row + 1];
        if constexpr (NEED_LAB) lab = a.labels[row];
    }
    for (; sv < a.nrows; sv = svn, row = rown, b = bn, e = en, lab = labn) {
        svn = sv + nwaves;
        rown = row;
        if (svn < a.nrows) rown = a.S ? a.S[svn] : svn;
        bn = a.rowptr[rown];
        en = a.rowptr[rown + 1];
        if constexpr (NEED_LAB) labn = a.labels[rown];
        T z;
        if constexpr (SPLIT) {
            const int64_t per = ((e - b + ROWS_WAVES_PER_BLOCK * NS - 1) / (ROWS_WAVES_PER_BLOCK * NS)) * NS;
            const int64_t wb = (b + wib * per < e) ? b + wib * per : e, we = (wb + per < e) ? wb + per : e;
            T *zp = zs + par * (ROWS_WAVES_PER_BLOCK * 64);
            zp[wib * 64 + lane] = csr_row_margin<T>(a, wb, we, lane, K, NS);
            __syncthreads();
            z = (zp[lane] + zp[64 + lane]) + (zp[128 + lane] + zp[192 + lane]);
            par ^= 1;
        } else {
            z = csr_row_margin<T>(a, b, e, lane, K, NS);
        }
        if constexpr (MODE == ROW_MARGIN) {              // margins of both operands, [X M | X M2], 2K values per row
            RowsArgs b2 = a;
            b2.M = a.M2;
            const T z2 = csr_row_margin<T>(b2, b, e, lane, K, NS);
            if (cv) {
                ((T *)a.UP)[sv * a.KP + lane] = z;
                ((T *)a.UP)[sv * a.KP + K + lane] = z2;
            }
            continue;
        }
        if constexpr (MODE == ROW_APPLY) {
            const T pin = cv ? ((const T *)a.Pin)[sv * a.KP + lane] : T(0);
            const T t = (K == 1) ? pin * z : wave_sum(pin * z);       // one weight column: lane 0 has it all
            const T u = pin * z - pin * t;
            if (cv) ((T *)a.UP)[sv * a.KP + lane] = u;
            // z_i . u_i of the row: summed over the sample it is V^T (X_S^T U), the curvature term CG needs
            const T zu = (K == 1) ? z * u : wave_sum(cv ? z * u : T(0));
            if (lane == 0) loss += (double)zu;
            continue;
        }
        // one weight column: the row's margin sits in lane 0 and nothing has to be reduced over the wave
        const T zmax = (K == 1) ? __shfl(z, 0) : wave_max(cv ? z : NEG);
        if constexpr (MODE == ROW_PRED) {
            const int cand = wave_min_int((cv && z == zmax) ? lane : 0x7fffffff);
            const int pr = (T(0) > zmax) ? K : cand;
            if (lane == 0) {
                if (a.pred) a.pred[sv] = pr;
                hits += (pr == lab);
            }
            continue;
        }
        const T Mx = fmax(T(0), zmax);
        const T ex = cv ? c_exp(z - Mx) : T(0);
        const T alpha = c_exp(-Mx) + ((K == 1) ? __shfl(ex, 0) : wave_sum(ex));
        if constexpr (MODE == ROW_PREP) {
            if (cv) ((T *)a.UP)[sv * a.KP + lane] = ex / alpha;
            continue;
        }
        const T lin = (K == 1) ? ((lab == 0) ? zmax : T(0)) : wave_sum((cv && lane == lab) ? z : T(0));
        if (lane == 0) loss += (double)Mx + (double)c_log(alpha) - (double)lin;
        if (MODE == ROW_GRAD && cv) ((T *)a.UP)[sv * a.KP + lane] = ex / alpha - ((lane == lab) ? T(1) : T(0));
    }
    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
        if (lane == 0) a.loss_part[wave] = loss;
    } else if constexpr (MODE == ROW_PRED) {
        if (lane == 0) a.hit_part[wave] = hits;
    }
}

// One weight column (the binary problem): a row's margin is a single number, and the per-row work on it (two
// exponentials, a logarithm, a division in eqs. (8), (9), (14)-(17)) done row by row keeps all 64 lanes busy with
// one row's arithmetic -- on rows of a few dozen entries that arithmetic, not the memory, is what the pass costs.
// Here a wave parks the margins of its rows in its lanes, one row per lane, and does the per-row work for up to 64
// rows at once.  Margins, prefetch and partial sums as in csr_rows_kernel; the loss of a wave is the sum of its lanes'
// sums (fixed order).
template <typename T, int MODE> __global__ __launch_bounds__(64 * ROWS_WAVES_PER_BLOCK) void csr_rows1_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const int64_t nwaves = (int64_t)gridDim.x * ROWS_WAVES_PER_BLOCK;
    const int64_t wave = (int64_t)blockIdx.x * ROWS_WAVES_PER_BLOCK + wib;
    double loss = 0.0;
    int hits = 0;
    // parked rows: lane i holds the margin, sample position and label of the i-th row since the last flush
    T zl = T(0);
    int64_t svl = 0;
    int labl = 0, cnt = 0;
    auto flush = [&]() {
        if (lane < cnt) {
            if constexpr (MODE == ROW_APPLY) {
                const T pin = ((const T *)a.Pin)[svl * a.KP];
                const T t = pin * zl;
                const T u = pin * zl - pin * t;              // eq. (12) with one class
                ((T *)a.UP)[svl * a.KP] = u;
                loss += (double)(zl * u);                    // z_i u_i: the curvature term of Alg. 2
            } else if constexpr (MODE == ROW_PRED) {
                const int pr = (T(0) > zl) ? 1 : 0;          // the reference class wins only strictly
                if (a.pred) a.pred[svl] = pr;
                hits += (pr == labl);
            } else {
                const T Mx = fmax(T(0), zl);
                const T ex = c_exp(zl - Mx);
                const T alpha = c_exp(-Mx) + ex;
                if constexpr (MODE == ROW_PREP) {
                    ((T *)a.UP)[svl * a.KP] = ex / alpha;
                } else {
                    loss += (double)Mx + (double)c_log(alpha) - (double)((labl == 0) ? zl : T(0));
                    if constexpr (MODE == ROW_GRAD) ((T *)a.UP)[svl * a.KP] = ex / alpha - ((labl == 0) ? T(1) : T(0));
                }
            }
        }
        cnt = 0;
    };

    int64_t sv = wave, svn = 0, row = 0, rown = 0, b = 0, e = 0, bn = 0, en = 0;
    int lab = 0, labn = 0;
    constexpr bool NEED_LAB = (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_PRED);
    if (sv < a.nrows) {
        row = a.S ? a.S[sv] : sv;
        b = a.rowptr[row];
        e = a.rowptr[row + 1];
        if constexpr (NEED_LAB) lab = a.labels[row];
    }
    for (; sv < a.nrows; sv = svn, row = rown, b = bn, e = en, lab = labn) {
        svn = sv + nwaves;
        rown = row;
        if (svn < a.nrows) rown = a.S ? a.S[svn] : svn;
        bn = a.rowptr[rown];
        en = a.rowptr[rown + 1];
        if constexpr (NEED_LAB) labn = a.labels[rown];
        const T z = __shfl(csr_row_margin<T>(a, b, e, lane, 1, 64), 0);
        if (lane == cnt) {
            zl = z;
            svl = sv;
            labl = lab;
        }
        if (++cnt == 64) flush();
    }
    flush();
    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
        loss = wave_sum(loss);
        if (lane == 0) a.loss_part[wave] = loss;
    } else if constexpr (MODE == ROW_PRED) {
        for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
        if (lane == 0) a.hit_part[wave] = hits;
    }
}

// One weight column, passes over ALL rows of the matrix: a lane per stored ENTRY instead of a wave per row.  A row of
// a few dozen entries gives a wave one short, dependent chain (pointers -> entries -> weights -> sum) and leaves half
// its lanes idle; here a wave takes an aligned window of 64 consecutive entries of the CSR arrays -- coalesced, no
// pointer chasing: the row of the window's first entry comes from an index built once (csr_window_rows_kernel).  The
// products x_e w_col are added up along the wave by an inclusive scan on the vector units (lane shifts inside rows of
// 16 lanes, then the two row broadcasts: no LDS traffic); then the lanes change roles -- lane j stands for row r0 + j,
// reads that row's first and last entry from the row pointers (coalesced), and takes the row's sum inside the window
// as the difference of two scan values fetched from the lanes of its last entry and of the entry before its first
// (the scan runs in fp64 whatever the data's precision, so the difference costs the sum nothing that shows).  A row that begins in the window leaves its
// sum in zrow[row] (coalesced), the leading part of a row that began in an earlier window goes to zhead[window];
// csr1_rowwork_kernel adds a row's pieces (its own, then the leading sums of the windows it runs into, in window
// order) and does the per-row work of eqs. (8), (9), (14)-(17) with a lane per row.  Windows that more than 64 rows
// reach into (runs of empty or one-entry rows) take the rows 64 at a time.
__global__ __launch_bounds__(256) void csr_window_rows_kernel(const int32_t *rowptr, int64_t n, int64_t nwin, int32_t *rwin)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= nwin) return;
    const int64_t target = w * 64;
    int64_t lo = 0, hi = n;                                  // rowptr[lo] <= target < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= target) lo = mid;
        else hi = mid;
    }
    rwin[w] = (int32_t)lo;
}

hipError_t launch_csr_window_rows(const int32_t *rowptr, int64_t n, int64_t nnz, int32_t *rwin, hipStream_t st)
{
    const int64_t nwin = (nnz + 63) / 64;
    if (nwin < 1 || n < 1) return hipSuccess;
    hipLaunchKernelGGL(csr_window_rows_kernel, dim3((unsigned)((nwin + 255) / 256)), dim3(256), 0, st, rowptr, n, nwin, rwin);
    return hipGetLastError();
}

// (a wave takes FLAT_WINDOWS consecutive windows and requests the entries, row pointers and weights of all of them
// before it works on the first: a single window is 768 bytes, far too little to have on the way per wave)
constexpr int FLAT_WINDOWS = 4;
template <typename T> __global__ __launch_bounds__(256) void csr1_flat_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    const int lane = threadIdx.x & 63;
    const int64_t w0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * FLAT_WINDOWS;
    if (w0 * 64 >= a.nnz) return;                                // the whole wave
    int col[FLAT_WINDOWS], r0[FLAT_WINDOWS], rs[FLAT_WINDOWS], re[FLAT_WINDOWS];
    T v[FLAT_WINDOWS], m[FLAT_WINDOWS];
#pragma unroll
    for (int i = 0; i < FLAT_WINDOWS; ++i) {
        const int64_t w = w0 + i, eg64 = w * 64 + lane;
        const bool have = eg64 < a.nnz;
        col[i] = have ? a.colidx[eg64] : 0;
        v[i] = have ? ((const T *)a.vals)[eg64] : T(0);
        r0[i] = (w * 64 < a.nnz) ? a.rwin[w] : 0;
    }
#pragma unroll
    for (int i = 0; i < FLAT_WINDOWS; ++i) {
        const int64_t r = (int64_t)r0[i] + lane;                 // this lane's row in its second role
        rs[i] = a.rowptr[r < a.n ? r : a.n];                     // (the entry count behind the last row)
        re[i] = a.rowptr[r + 1 < a.n ? r + 1 : a.n];
        m[i] = ((const T *)a.M)[(int64_t)col[i] * a.ldm];
    }
#pragma unroll
    for (int i = 0; i < FLAT_WINDOWS; ++i) {
        const int64_t w = w0 + i;
        if (w * 64 >= a.nnz) break;                              // the whole wave
        const int wbeg = (int)(w * 64);                          // entry counts fit 31 bits
        const int wend = (a.nnz - wbeg < 64) ? (int)a.nnz : wbeg + 64;
        // (the scan runs in fp64 in both precisions: a difference of two fp32 prefix sums would lose the bits that
        // the sums before the row have used up, and the line search near convergence compares objectives to the last)
        const double P = wave_inclusive_scan((wbeg + lane < wend) ? (double)v[i] * (double)m[i] : 0.0);
        int rsl = rs[i], rel = re[i];
        for (int64_t base = r0[i];;) {
            const int b = (rsl > wbeg ? rsl : wbeg) - wbeg, e = (rel < wend ? rel : wend) - wbeg;
            const double Pe = __shfl(P, e > 0 ? e - 1 : 0), Pb = __shfl(P, b > 0 ? b - 1 : 0);
            if (base + lane < a.n && e > b) {
                const T sum = (T)((b > 0) ? Pe - Pb : Pe);
                if (rsl < wbeg) ((T *)a.zhead)[w] = sum;         // (lane 0 of the first 64 rows only)
                else ((T *)a.zrow)[base + lane] = sum;
            }
            if (base == r0[i] && lane == 0 && !(rsl < wbeg)) ((T *)a.zhead)[w] = T(0);
            // the rows behind these 64 reach into the window too?
            const int last_end = __shfl(rel, 63);
            base += 64;
            if (last_end >= wend || base >= a.n) break;          // uniform over the wave
            const int64_t r = base + lane;
            rsl = a.rowptr[r < a.n ? r : a.n];
            rel = a.rowptr[r + 1 < a.n ? r + 1 : a.n];
        }
    }
}

template <typename T, int MODE> __global__ __launch_bounds__(256) void csr1_rowwork_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * ROWS_WAVES_PER_BLOCK + (threadIdx.x >> 6);
    double loss = 0.0;
    int hits = 0;
    const T *zrow = (const T *)a.zrow, *zhead = (const T *)a.zhead;
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < a.n; r += (int64_t)gridDim.x * 256) {
        const int b = a.rowptr[r], e = a.rowptr[r + 1];
        const int lab = a.labels[r];
        T z = T(0);
        if (e > b) {
            z = zrow[r];
            for (int w2 = b / 64 + 1; w2 <= (e - 1) / 64; ++w2) z += zhead[w2];
        }
        if constexpr (MODE == ROW_PRED) {
            const int pr = (T(0) > z) ? 1 : 0;                   // the reference class wins only strictly
            if (a.pred) a.pred[r] = pr;
            hits += (pr == lab);
        } else {
            const T Mx = fmax(T(0), z);
            const T ex = c_exp(z - Mx);
            const T alpha = c_exp(-Mx) + ex;
            loss += (double)Mx + (double)c_log(alpha) - (double)((lab == 0) ? z : T(0));
            if constexpr (MODE == ROW_GRAD) ((T *)a.UP)[r * a.KP] = ex / alpha - ((lab == 0) ? T(1) : T(0));
        }
    }
    if constexpr (MODE == ROW_PRED) {
        for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
        if (lane == 0) a.hit_part[wave] = hits;
    } else {
        loss = wave_sum(loss);
        if (lane == 0) a.loss_part[wave] = loss;
    }
}

template <typename T> static hipError_t csr_rows_dispatch(const RowsArgs &a, int blocks, hipStream_t st)
{
    dim3 grid(blocks), block(64 * ROWS_WAVES_PER_BLOCK);
    if (a.K == 1 && a.rwin && !a.S && a.nnz > 0 && (a.mode == ROW_OBJ || a.mode == ROW_GRAD || a.mode == ROW_PRED)) {
        const unsigned fblocks = (unsigned)((((a.nnz + 63) / 64) + 4 * FLAT_WINDOWS - 1) / (4 * FLAT_WINDOWS));
        hipLaunchKernelGGL(csr1_flat_kernel<T>, dim3(fblocks), dim3(256), 0, st, a);
        switch (a.mode) {
        case ROW_OBJ: hipLaunchKernelGGL((csr1_rowwork_kernel<T, ROW_OBJ>), grid, block, 0, st, a); break;
        case ROW_GRAD: hipLaunchKernelGGL((csr1_rowwork_kernel<T, ROW_GRAD>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((csr1_rowwork_kernel<T, ROW_PRED>), grid, block, 0, st, a); break;
        }
        return hipGetLastError();
    }
    if (a.K == 1) {                      // one weight column: per-row work for up to 64 rows at once
        switch (a.mode) {
        case ROW_OBJ: hipLaunchKernelGGL((csr_rows1_kernel<T, ROW_OBJ>), grid, block, 0, st, a); return hipGetLastError();
        case ROW_GRAD: hipLaunchKernelGGL((csr_rows1_kernel<T, ROW_GRAD>), grid, block, 0, st, a); return hipGetLastError();
        case ROW_PREP: hipLaunchKernelGGL((csr_rows1_kernel<T, ROW_PREP>), grid, block, 0, st, a); return hipGetLastError();
        case ROW_APPLY: hipLaunchKernelGGL((csr_rows1_kernel<T, ROW_APPLY>), grid, block, 0, st, a); return hipGetLastError();
        case ROW_PRED: hipLaunchKernelGGL((csr_rows1_kernel<T, ROW_PRED>), grid, block, 0, st, a); return hipGetLastError();
        default: break;                  // ROW_MARGIN: the general kernel
        }
    }
    if (a.csr_split) {                   // a workgroup per row (the launcher asks for it on the modes below only)
        switch (a.mode) {
        case ROW_PREP: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_PREP, true>), grid, block, 0, st, a); return hipGetLastError();
        case ROW_APPLY: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_APPLY, true>), grid, block, 0, st, a); return hipGetLastError();
        default: return hipErrorInvalidValue;
        }
    }
    switch (a.mode) {
    case ROW_OBJ: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_OBJ>), grid, block, 0, st, a); break;
    case ROW_GRAD: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_GRAD>), grid, block, 0, st, a); break;
    case ROW_PREP: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_PREP>), grid, block, 0, st, a); break;
    case ROW_APPLY: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_APPLY>), grid, block, 0, st, a); break;
    case ROW_PRED: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_PRED>), grid, block, 0, st, a); break;
    case ROW_MARGIN: hipLaunchKernelGGL((csr_rows_kernel<T, ROW_MARGIN>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_csr_rows(int dtype, const RowsArgs &a, int blocks, hipStream_t st)
{
    return dtype == SSN_F32 ? csr_rows_dispatch<float>(a, blocks, st) : csr_rows_dispatch<double>(a, blocks, st);
}

}  // namespace ssn
