// Dense kernels for the binary problem (C = 2, one weight column; Appendix A.1 of the paper shows it is plain
// logistic regression).  With K = 1 both products are matrix-vector products, z = X w and g = X^T u: there is no
// class dimension to tile, a 16-column matrix-core tile would be 15/16 padding, and one multiply-add per element
// of X is far below what the vector units deliver at HBM speed.  So these are GEMV-shaped kernels on the vector
// units:
//   rows kernel : a wave owns two rows at a time and walks their features with 16-byte loads, eight per row in
//                 flight; z_i is a wave reduction; the per-row work of eqs. (8), (9), (14)-(17) / eq. (12)
//                 (K = 1: u = p (1 - p) z) is a handful of scalar operations per row;
//   xtu kernel  : part[chunk][j] = sum over the chunk's rows of x_ij u_i, a thread per 16 bytes of features,
//                 rows eight at a time, u_i uniform over the block; the chunk partials are added by the
//                 finalize kernels of the general path (fixed order, no atomics).
// Per-row buffers (U, P) have row stride a.KP (1 on this path).
#include "ssn_internal.h"
#include "ssn_math.h"

namespace ssn {

namespace {

__device__ __forceinline__ float b_exp(float x) { return expf(x); }
__device__ __forceinline__ double b_exp(double x) { return exp_nonpos(x, 0.0); }
__device__ __forceinline__ float b_log(float x) { return logf(x); }
__device__ __forceinline__ double b_log(double x) { return log_ge1(x); }

template <typename T, int VEC> struct alignas(sizeof(T) * VEC) BPack { T v[VEC]; };

template <typename T> __device__ __forceinline__ T wave_sum64(T x)
{
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// per-row work for margin z of sample position sv (all lanes hold the same values)
template <typename T, int MODE>
__device__ __forceinline__ void binary_row(const RowsArgs &a, int64_t sv, int64_t row, T z, int lane, double &loss, int &hits)
{
    if constexpr (MODE == ROW_APPLY) {
        const T pin = ((const T *)a.Pin)[sv * a.KP];
        const T t = pin * z;
        const T u = pin * z - pin * t;                     // eq. (12) with one class
        if (lane == 0) {
            ((T *)a.UP)[sv * a.KP] = u;
            loss += (double)(z * u);                       // z_i u_i: the curvature term of Alg. 2
        }
        return;
    }
    if constexpr (MODE == ROW_PRED) {
        const int pr = (T(0) > z) ? 1 : 0;                 // the reference class wins only strictly
        if (lane == 0) {
            if (a.pred) a.pred[sv] = pr;
            hits += (pr == a.labels[row]);
        }
        return;
    }
    // eqs. (8), (9): M = max{0, z}, alpha = e^{-M} + e^{z - M}
    const T Mx = fmax(T(0), z);
    const T e = b_exp(z - Mx);
    const T alpha = b_exp(-Mx) + e;
    if constexpr (MODE == ROW_PREP) {
        if (lane == 0) ((T *)a.UP)[sv * a.KP] = e / alpha;
        return;
    }
    const int lab = a.labels[row];
    if (lane == 0) {
        loss += (double)Mx + (double)b_log(alpha) - (double)((lab == 0) ? z : T(0));      // eqs. (14)-(17)
        if constexpr (MODE == ROW_GRAD) ((T *)a.UP)[sv * a.KP] = e / alpha - ((lab == 0) ? T(1) : T(0));
    }
}

template <typename T, int VEC, int MODE> __global__ __launch_bounds__(256) void binary_rows_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef BPack<T, VEC> pack;
    constexpr int UNR = 8;                   // vector loads per row in flight
    const int lane = threadIdx.x & 63;
    const int64_t nwaves = (int64_t)gridDim.x * 4, wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const T *X = (const T *)a.X;
    const T *w = (const T *)a.M;             // p weights, stride a.ldm
    // ROW_MARGIN: the margins of a second operand ride along (the same loads of X serve both)
    constexpr bool TWO = MODE == ROW_MARGIN;
    const T *w2 = TWO ? (const T *)a.M2 : w;
    const int64_t p = a.p, ldm = a.ldm;
    const int64_t pv = p / VEC * VEC;        // features covered by whole vectors
    double loss = 0.0;
    int hits = 0;
    for (int64_t s0 = wave * 2; s0 < a.nrows; s0 += nwaves * 2) {
        const bool two = s0 + 1 < a.nrows;
        const int64_t s1 = two ? s0 + 1 : s0;
        const int64_t r0 = a.S ? (int64_t)a.S[s0] : s0, r1 = a.S ? (int64_t)a.S[s1] : s1;
        const T *x0 = X + r0 * a.ldx, *x1 = X + r1 * a.ldx;
        T z0 = 0, z1 = 0, y0 = 0, y1 = 0;
        int64_t f = (int64_t)lane * VEC;
        for (; f + (int64_t)(UNR - 1) * 64 * VEC < pv; f += (int64_t)UNR * 64 * VEC) {
            pack xa[UNR], xb[UNR];
            T wv[UNR][VEC];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                xa[u] = *(const pack *)(x0 + f + (int64_t)u * 64 * VEC);
                xb[u] = *(const pack *)(x1 + f + (int64_t)u * 64 * VEC);
#pragma unroll
                for (int m = 0; m < VEC; ++m) wv[u][m] = w[(f + (int64_t)u * 64 * VEC + m) * ldm];
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int m = 0; m < VEC; ++m) {
                    z0 += xa[u].v[m] * wv[u][m];
                    z1 += xb[u].v[m] * wv[u][m];
                    if constexpr (TWO) {
                        const T w2m = w2[(f + (int64_t)u * 64 * VEC + m) * ldm];
                        y0 += xa[u].v[m] * w2m;
                        y1 += xb[u].v[m] * w2m;
                    }
                }
        }
        for (; f < pv; f += 64 * VEC) {
            const pack xa = *(const pack *)(x0 + f), xb = *(const pack *)(x1 + f);
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const T wm = w[(f + m) * ldm];
                z0 += xa.v[m] * wm;
                z1 += xb.v[m] * wm;
                if constexpr (TWO) {
                    const T w2m = w2[(f + m) * ldm];
                    y0 += xa.v[m] * w2m;
                    y1 += xb.v[m] * w2m;
                }
            }
        }
        for (int64_t g = pv + lane; g < p; g += 64) {          // features beyond the last whole vector
            const T wm = w[g * ldm];
            z0 += x0[g] * wm;
            z1 += x1[g] * wm;
            if constexpr (TWO) {
                const T w2m = w2[g * ldm];
                y0 += x0[g] * w2m;
                y1 += x1[g] * w2m;
            }
        }
        z0 = wave_sum64(z0);
        z1 = wave_sum64(z1);
        if constexpr (TWO) {                 // [x.w, x.w2] per row
            y0 = wave_sum64(y0);
            y1 = wave_sum64(y1);
            if (lane == 0) {
                T *Z = (T *)a.UP;
                Z[s0 * a.KP] = z0;
                Z[s0 * a.KP + 1] = y0;
                if (two) {
                    Z[s1 * a.KP] = z1;
                    Z[s1 * a.KP + 1] = y1;
                }
            }
            continue;
        }
        binary_row<T, MODE>(a, s0, r0, z0, lane, loss, hits);
        if (two) binary_row<T, MODE>(a, s1, r1, z1, lane, loss, hits);
    }
    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
        if (lane == 0) a.loss_part[wave] = loss;
    } else if constexpr (MODE == ROW_PRED) {
        if (lane == 0) a.hit_part[wave] = hits;
    }
}

// grid: (feature tiles of 256 * VEC, row chunks)
template <typename T, int VEC> __global__ __launch_bounds__(256) void binary_xtu_kernel(XtuArgs a)
{
    if (a.skip && *a.skip) return;
    typedef BPack<T, VEC> pack;
    constexpr int RU = 8;
    const int64_t f = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (f >= a.p) return;
    const int64_t chunk = blockIdx.y;
    const int64_t r_begin = chunk * a.rows_per_chunk;
    const int64_t r_end = min(a.nrows, r_begin + a.rows_per_chunk);
    const T *X = (const T *)a.X;
    const T *U = (const T *)a.U;
    const bool whole = f + VEC <= a.p;
    T acc[VEC];
#pragma unroll
    for (int m = 0; m < VEC; ++m) acc[m] = 0;
    int64_t r = r_begin;
    if (whole) {
        for (; r + RU <= r_end; r += RU) {
            pack xv[RU];
            T u[RU];
#pragma unroll
            for (int k = 0; k < RU; ++k) {
                const int64_t xr = a.S ? (int64_t)a.S[r + k] : r + k;
                xv[k] = *(const pack *)(X + xr * a.ldx + f);
                u[k] = U[(r + k) * a.KP];
            }
#pragma unroll
            for (int k = 0; k < RU; ++k)
#pragma unroll
                for (int m = 0; m < VEC; ++m) acc[m] += xv[k].v[m] * u[k];
        }
    }
    for (; r < r_end; ++r) {
        const int64_t xr = a.S ? (int64_t)a.S[r] : r;
        const T u = U[r * a.KP];
#pragma unroll
        for (int m = 0; m < VEC; ++m)
            if (f + m < a.p) acc[m] += X[xr * a.ldx + f + m] * u;
    }
    T *part = (T *)a.part + chunk * a.p;                    // K = 1: a chunk's partial is p elements
#pragma unroll
    for (int m = 0; m < VEC; ++m)
        if (f + m < a.p) part[f + m] = acc[m];
}

template <typename T, int VEC> hipError_t rows_mode(const RowsArgs &a, int blocks, hipStream_t st)
{
    dim3 grid(blocks), block(256);
    switch (a.mode) {
    case ROW_OBJ: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_OBJ>), grid, block, 0, st, a); break;
    case ROW_GRAD: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_GRAD>), grid, block, 0, st, a); break;
    case ROW_PREP: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_PREP>), grid, block, 0, st, a); break;
    case ROW_APPLY: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_APPLY>), grid, block, 0, st, a); break;
    case ROW_PRED: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_PRED>), grid, block, 0, st, a); break;
    case ROW_MARGIN: hipLaunchKernelGGL((binary_rows_kernel<T, VEC, ROW_MARGIN>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T> bool rows_aligned(const void *X, int64_t ldx)
{
    return ((uintptr_t)X % 16 == 0) && ((ldx * (int64_t)sizeof(T)) % 16 == 0);
}

}  // namespace

// workgroups (4 waves each, one loss / hit partial per wave) for a pass over nrows rows, two rows per wave and trip
int binary_rows_blocks(int64_t nrows, int num_cus)
{
    int64_t b = (nrows + 7) / 8;
    const int64_t cap = (int64_t)num_cus * 8;
    if (b > cap) b = cap;
    return (int)(b < 1 ? 1 : b);
}

hipError_t launch_binary_rows(int dtype, const RowsArgs &a, int blocks, hipStream_t st)
{
    if (a.K != 1) return hipErrorInvalidValue;
    if (dtype == SSN_F32)
        return rows_aligned<float>(a.X, a.ldx) ? rows_mode<float, 4>(a, blocks, st) : rows_mode<float, 1>(a, blocks, st);
    return rows_aligned<double>(a.X, a.ldx) ? rows_mode<double, 2>(a, blocks, st) : rows_mode<double, 1>(a, blocks, st);
}

hipError_t launch_binary_xtu(int dtype, const XtuArgs &a, hipStream_t st)
{
    if (a.K != 1) return hipErrorInvalidValue;
    if (dtype == SSN_F32) {
        if (rows_aligned<float>(a.X, a.ldx)) {
            dim3 grid((unsigned)((a.p + 1023) / 1024), (unsigned)a.nchunks);
            hipLaunchKernelGGL((binary_xtu_kernel<float, 4>), grid, dim3(256), 0, st, a);
        } else {
            dim3 grid((unsigned)((a.p + 255) / 256), (unsigned)a.nchunks);
            hipLaunchKernelGGL((binary_xtu_kernel<float, 1>), grid, dim3(256), 0, st, a);
        }
    } else {
        if (rows_aligned<double>(a.X, a.ldx)) {
            dim3 grid((unsigned)((a.p + 511) / 512), (unsigned)a.nchunks);
            hipLaunchKernelGGL((binary_xtu_kernel<double, 2>), grid, dim3(256), 0, st, a);
        } else {
            dim3 grid((unsigned)((a.p + 255) / 256), (unsigned)a.nchunks);
            hipLaunchKernelGGL((binary_xtu_kernel<double, 1>), grid, dim3(256), 0, st, a);
        }
    }
    return hipGetLastError();
}

}  // namespace ssn
