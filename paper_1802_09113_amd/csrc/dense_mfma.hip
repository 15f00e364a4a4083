// Dense row-major kernels on the gfx950 matrix cores.
//
// Both products of the method are tall-and-skinny contractions against a K-column block
// (K = C-1 <= 32, padded to 16-column MFMA tiles):
//   rows kernel : Z = X_rows * M   (Alg. 5 l.3, Alg. 6 l.3, Alg. 7 l.3) with the per-row work of
//                 Alg. 4 / eq. (8),(9),(14)-(17) / Alg. 8 fused in as an epilogue on the MFMA
//                 accumulators, so the n x K margin matrix never goes to memory;
//   xtu kernel  : part = X_rows^T * U (Alg. 6 l.4, Alg. 7 l.6) as per-row-chunk partial sums that a
//                 finalize kernel adds in a fixed order (deterministic, no atomics).
//
// MFMA tile used throughout: v_mfma_{f32,f64}_16x16x4 -- D(16x16) += A(16x4) * B(4x16), wave64:
//   lane l supplies A[l%16][l/16] and B[l/16][l%16]; accumulator element v (0..3) of lane l is
//   D[4*(l/16)+v][l%16] for the f32 instruction and D[4*v+l/16][l%16] for the f64 one (d_row below).
#include "ssn_internal.h"

#include <limits>

namespace ssn {

template <typename T> struct V4;
template <> struct V4<float> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct V4<double> { typedef double type __attribute__((ext_vector_type(4))); };

__device__ __forceinline__ V4<double>::type mfma16(double a, double b, V4<double>::type c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ V4<float>::type mfma16(float a, float b, V4<float>::type c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// row of the 16x16 output tile held in accumulator element v of a lane in 16-lane group g
template <typename T> __device__ __forceinline__ int d_row(int g, int v);
template <> __device__ __forceinline__ int d_row<float>(int g, int v) { return 4 * g + v; }
template <> __device__ __forceinline__ int d_row<double>(int g, int v) { return 4 * v + g; }

template <typename T, int VEC> struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };

__device__ __forceinline__ float t_exp(float x) { return expf(x); }
__device__ __forceinline__ double t_exp(double x) { return exp(x); }
__device__ __forceinline__ float t_log(float x) { return logf(x); }
__device__ __forceinline__ double t_log(double x) { return log(x); }

// butterfly over the 16 lanes that hold the 16 class columns of one row
template <typename T> __device__ __forceinline__ T row16_sum(T x)
{
    x += __shfl_xor(x, 8);
    x += __shfl_xor(x, 4);
    x += __shfl_xor(x, 2);
    x += __shfl_xor(x, 1);
    return x;
}
template <typename T> __device__ __forceinline__ T row16_max(T x)
{
    x = fmax(x, __shfl_xor(x, 8));
    x = fmax(x, __shfl_xor(x, 4));
    x = fmax(x, __shfl_xor(x, 2));
    x = fmax(x, __shfl_xor(x, 1));
    return x;
}
__device__ __forceinline__ int row16_min(int x)
{
    x = min(x, __shfl_xor(x, 8));
    x = min(x, __shfl_xor(x, 4));
    x = min(x, __shfl_xor(x, 2));
    x = min(x, __shfl_xor(x, 1));
    return x;
}

// Per-row work on a 16-row block of margins held in MFMA accumulator layout:
// acc[nb][v] = z(row d_row<T>(lane/16, v), class 16*nb + lane%16).
// TOREG: U (ROW_GRAD / ROW_APPLY) is returned in `uout` in the same accumulator layout instead of being
// stored.  vmask selects which of the 4 accumulator elements (row groups) this wave works on.
template <typename T, int NB, int MODE, bool TOREG = false>
__device__ __forceinline__ void row_epilogue(const typename V4<T>::type (&acc)[NB], const RowsArgs &a,
                                             int64_t rb, int lane, double &loss, int &hits,
                                             typename V4<T>::type *uout = nullptr, int vmask = 15,
                                             const int *lab_pre = nullptr, const T *pin_pre = nullptr)
{
    // lab_pre / pin_pre (one-pass kernel, NB == 1): label and probability of each accumulator element,
    // loaded by the caller ahead of its X prefetch so that waiting for them does not drain that prefetch
    constexpr bool primary = true;
    const int q = lane & 15, g = lane >> 4;
    const int K = a.K;
    const T NEG = -std::numeric_limits<T>::infinity();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (!((vmask >> v) & 1)) continue;
        const int64_t sv = rb * 16 + d_row<T>(g, v);
        const bool valid = sv < a.nrows;
        const int64_t svc = valid ? sv : a.nrows - 1;
        T z[NB];
        bool cv[NB];
        T zmax = NEG;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            cv[nb] = (nb * 16 + q) < K;
            z[nb] = acc[nb][v];
            zmax = fmax(zmax, cv[nb] ? z[nb] : NEG);
        }
        zmax = row16_max(zmax);
        if constexpr (MODE == ROW_PRED) {
            int lab;
            if (lab_pre) lab = lab_pre[v];
            else lab = a.labels[a.S ? a.S[svc] : svc];
            int cand = 0x7fffffff;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                if (cv[nb] && z[nb] == zmax) cand = min(cand, nb * 16 + q);
            cand = row16_min(cand);
            const int pr = (T(0) > zmax) ? K : cand;     // the reference class wins only strictly
            if (primary && valid && q == 0) {
                if (a.pred) a.pred[sv] = pr;
                hits += (pr == lab);
            }
            continue;
        }
        if constexpr (MODE == ROW_APPLY) {
            // eq. (12): u = p .* vhat - p * <p, vhat>
            const T *Pin = (const T *)a.Pin;
            T pin[NB];
            T t = 0;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                pin[nb] = pin_pre ? pin_pre[v] : Pin[svc * a.KP + nb * 16 + q];      // zero in padded columns
                t += pin[nb] * z[nb];
            }
            t = row16_sum(t);
            T *U = (T *)a.UP;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const T u = valid ? (pin[nb] * z[nb] - pin[nb] * t) : T(0);
                if constexpr (TOREG) uout[nb][v] = u;
                else U[sv * a.KP + nb * 16 + q] = u;
            }
            continue;
        }
        // eq. (8), (9): M = max{0, z}, alpha = e^{-M} + sum_c e^{z_c - M}
        const T Mx = fmax(T(0), zmax);
        T e[NB];
        T se = 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            e[nb] = cv[nb] ? t_exp(z[nb] - Mx) : T(0);
            se += e[nb];
        }
        se = row16_sum(se);
        const T alpha = t_exp(-Mx) + se;
        if constexpr (MODE == ROW_PREP) {
            T *P = (T *)a.UP;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                if (primary) P[sv * a.KP + nb * 16 + q] = valid ? e[nb] / alpha : T(0);
            continue;
        }
        // ROW_OBJ / ROW_GRAD: eqs. (14)-(17)
        int lab;
        if (lab_pre) lab = lab_pre[v];
        else lab = a.labels[a.S ? a.S[svc] : svc];
        T lin = 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            lin += (cv[nb] && (nb * 16 + q) == lab) ? z[nb] : T(0);
        lin = row16_sum(lin);
        if (primary && valid && q == 0) loss += (double)Mx + (double)t_log(alpha) - (double)lin;
        if constexpr (MODE == ROW_GRAD) {
            T *U = (T *)a.UP;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const T ind = ((nb * 16 + q) == lab) ? T(1) : T(0);
                const T u = (valid && cv[nb]) ? (e[nb] / alpha - ind) : T(0);
                if constexpr (TOREG) uout[nb][v] = u;
                else U[sv * a.KP + nb * 16 + q] = u;
            }
        }
    }
}

// One wave per 16-row block; grid-stride over row blocks.  UP / Pin have ceil(nrows/16)*16 rows.
template <typename T, int NB, int VEC, int MODE>
__global__ __launch_bounds__(64 * ROWS_WAVES_PER_BLOCK) void dense_rows_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    typedef Pack<T, VEC> pack;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const int q = lane & 15, g = lane >> 4;
    const int64_t nwaves = (int64_t)gridDim.x * ROWS_WAVES_PER_BLOCK;
    const int64_t wave = (int64_t)blockIdx.x * ROWS_WAVES_PER_BLOCK + wib;
    const T *X = (const T *)a.X;
    const T *M = (const T *)a.M;
    const int K = a.K;
    const int64_t p = a.p, ldm = a.ldm;

    bool cval[NB];
    const T *mcol[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int c = nb * 16 + q;
        cval[nb] = c < K;
        mcol[nb] = M + (cval[nb] ? c : K - 1);
    }

    double loss = 0.0;
    int hits = 0;
    const int64_t nblk = (a.nrows + 15) / 16;
    constexpr int STEP = 4 * VEC;     // features consumed per vector load (4 k-groups of VEC)
    constexpr int UNR = 4;

    for (int64_t rb = wave; rb < nblk; rb += nwaves) {
        int64_t si = rb * 16 + q;
        if (si >= a.nrows) si = a.nrows - 1;          // clamped rows are masked in the epilogue
        const int64_t xr = a.S ? a.S[si] : si;
        const T *xrow = X + xr * a.ldx;
        v4 acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = v4{0, 0, 0, 0};

        int64_t f0 = 0;
        for (; f0 + STEP * UNR <= p; f0 += STEP * UNR) {
            pack xv[UNR];
            T wv[UNR][VEC][NB];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int64_t f = f0 + u * STEP + VEC * g;
                xv[u] = *(const pack *)(xrow + f);
#pragma unroll
                for (int m = 0; m < VEC; ++m)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) wv[u][m][nb] = mcol[nb][(f + m) * ldm];
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int m = 0; m < VEC; ++m)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb] = mfma16(xv[u].v[m], cval[nb] ? wv[u][m][nb] : T(0), acc[nb]);
        }
        for (; f0 < p; f0 += STEP) {                   // guarded tail
            const int64_t f = f0 + VEC * g;
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const bool ok = (f + m) < p;
                const T x = ok ? xrow[f + m] : T(0);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const T w = (ok && cval[nb]) ? mcol[nb][(f + m) * ldm] : T(0);
                    acc[nb] = mfma16(x, w, acc[nb]);
                }
            }
        }
        row_epilogue<T, NB, MODE>(acc, a, rb, lane, loss, hits);
    }

    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD) {
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
        if (lane == 0) a.loss_part[wave] = loss;
    } else if constexpr (MODE == ROW_PRED) {
        for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
        if (lane == 0) a.hit_part[wave] = hits;
    }
}

// part[chunk] (p x K) = sum over the chunk's rows of x_row^T u_row.
// Block = 4 waves, each wave owns 64 consecutive features; blockIdx.y = row chunk.
// A vector load of VEC consecutive features per lane feeds VEC MFMAs whose output rows are the
// features {base + VEC*i + m : i = 0..15}.
template <typename T, int NB, int VEC>
__global__ __launch_bounds__(256) void dense_xtu_kernel(XtuArgs a)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    typedef Pack<T, VEC> pack;
    constexpr int FT = 64;
    constexpr int NL = FT / (16 * VEC);
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const int q = lane & 15, g = lane >> 4;
    const int64_t p = a.p;
    const int K = a.K;
    const int64_t f0 = ((int64_t)blockIdx.x * 4 + wib) * FT;
    if (f0 >= p) return;
    const int64_t chunk = blockIdx.y;
    const int64_t r_begin = chunk * a.rows_per_chunk;
    const int64_t r_end = min(a.nrows, r_begin + a.rows_per_chunk);
    const T *X = (const T *)a.X;
    const T *U = (const T *)a.U;
    const bool full = (f0 + FT) <= p;

    v4 acc[NL * VEC][NB];
#pragma unroll
    for (int t = 0; t < NL * VEC; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = v4{0, 0, 0, 0};

    for (int64_t r0 = r_begin; r0 < r_end; r0 += 4) {
        const int64_t si = r0 + g;
        const bool rv = si < r_end;
        const int64_t sc = rv ? si : r_begin;
        const int64_t xr = a.S ? a.S[sc] : sc;
        const T *xrow = X + xr * a.ldx + f0;
        T ub[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const T u = U[sc * a.KP + nb * 16 + q];
            ub[nb] = rv ? u : T(0);
        }
#pragma unroll
        for (int ld = 0; ld < NL; ++ld) {
            const int fl = ld * 16 * VEC + VEC * q;
            pack xv;
            if (full) {
                xv = *(const pack *)(xrow + fl);
            } else {
#pragma unroll
                for (int m = 0; m < VEC; ++m) xv.v[m] = (f0 + fl + m) < p ? xrow[fl + m] : T(0);
            }
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const T x = rv ? xv.v[m] : T(0);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[ld * VEC + m][nb] = mfma16(x, ub[nb], acc[ld * VEC + m][nb]);
            }
        }
    }

    T *part = (T *)a.part + chunk * p * K;
#pragma unroll
    for (int ld = 0; ld < NL; ++ld)
#pragma unroll
        for (int m = 0; m < VEC; ++m)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int64_t f = f0 + ld * 16 * VEC + VEC * d_row<T>(g, v) + m;
                    const int c = nb * 16 + q;
                    if (f < p && c < K) part[f * K + c] = acc[ld * VEC + m][nb][v];
                }
}

int rows_grid_blocks(int64_t nrows, int num_cus)
{
    const int64_t nblk = (nrows + 15) / 16;
    int64_t blocks = (nblk + ROWS_WAVES_PER_BLOCK - 1) / ROWS_WAVES_PER_BLOCK;
    const int64_t cap = (int64_t)num_cus * 8;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

template <typename T> static bool vec_ok(const void *X, int64_t ldx)
{
    constexpr int VEC = 16 / sizeof(T);
    return ((uintptr_t)X % 16 == 0) && (ldx % VEC == 0);
}

template <typename T, int MODE> static hipError_t rows_dispatch_mode(const RowsArgs &a, int blocks, hipStream_t st)
{
    constexpr int VEC = 16 / sizeof(T);
    const int nb = (a.K + 15) / 16;
    const bool v = vec_ok<T>(a.X, a.ldx);
    dim3 grid(blocks), block(64 * ROWS_WAVES_PER_BLOCK);
    if (nb == 1) {
        if (v) hipLaunchKernelGGL((dense_rows_kernel<T, 1, VEC, MODE>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_rows_kernel<T, 1, 1, MODE>), grid, block, 0, st, a);
    } else if (nb == 2) {
        if (v) hipLaunchKernelGGL((dense_rows_kernel<T, 2, VEC, MODE>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_rows_kernel<T, 2, 1, MODE>), grid, block, 0, st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T> static hipError_t rows_dispatch(const RowsArgs &a, int blocks, hipStream_t st)
{
    switch (a.mode) {
    case ROW_OBJ: return rows_dispatch_mode<T, ROW_OBJ>(a, blocks, st);
    case ROW_GRAD: return rows_dispatch_mode<T, ROW_GRAD>(a, blocks, st);
    case ROW_PREP: return rows_dispatch_mode<T, ROW_PREP>(a, blocks, st);
    case ROW_APPLY: return rows_dispatch_mode<T, ROW_APPLY>(a, blocks, st);
    case ROW_PRED: return rows_dispatch_mode<T, ROW_PRED>(a, blocks, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_dense_rows(int dtype, const RowsArgs &a, int blocks, hipStream_t st)
{
    return dtype == SSN_F32 ? rows_dispatch<float>(a, blocks, st) : rows_dispatch<double>(a, blocks, st);
}

template <typename T> static hipError_t xtu_dispatch(const XtuArgs &a, hipStream_t st)
{
    constexpr int VEC = 16 / sizeof(T);
    const int nb = (a.K + 15) / 16;
    const bool v = vec_ok<T>(a.X, a.ldx);
    dim3 grid((unsigned)((a.p + 255) / 256), (unsigned)a.nchunks), block(256);
    if (nb == 1) {
        if (v) hipLaunchKernelGGL((dense_xtu_kernel<T, 1, VEC>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_xtu_kernel<T, 1, 1>), grid, block, 0, st, a);
    } else if (nb == 2) {
        if (v) hipLaunchKernelGGL((dense_xtu_kernel<T, 2, VEC>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_xtu_kernel<T, 2, 1>), grid, block, 0, st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dense_xtu(int dtype, const XtuArgs &a, hipStream_t st)
{
    return dtype == SSN_F32 ? xtu_dispatch<float>(a, st) : xtu_dispatch<double>(a, st);
}

// ---------------------------------------------------------------------------------------------
// Fused one-pass kernel: margins, per-row epilogue and (for ROW_GRAD / ROW_APPLY) the transposed
// product, reading every row of X exactly once (eqs. (10)-(13) with both products of Alg. 7 in one
// sweep; same for Alg. 6).
//
// A workgroup owns whole 16-row blocks; its waves split the features into slices of a.fw features
// (a.fw <= 16*NT, a multiple of the vector width).  Per row block:
//   1. every lane already holds its part of the wave's 16 x fw tile of X in the A-operand layout
//      (prefetched into registers while the previous block was processed);
//   2. phase A: Z_partial (16x16) += X_tile * W_slice, W operands from an LDS copy of M;
//   3. the partial margins of the waves are added through LDS in a fixed order (two barriers);
//   4. every wave runs the epilogue on the full margins and keeps U in accumulator layout, which is
//      exactly the B-operand layout of the transposed product;
//   5. phase C: the wave's X tile is transposed through a wave-private LDS scratch (rows become the
//      contraction index) and G_slice (fw x 16) += X_tile^T * U accumulates in registers.
// At the end each workgroup writes its p x K partial; the finalize kernel adds them in a fixed order.
template <typename T, int MODE, int NLD, int NSB>
__global__ __launch_bounds__(512) void dense_fused_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    constexpr int VEC = 16 / sizeof(T);
    typedef Pack<T, VEC> pack;
    // NLD: vector loads per lane per row block the instantiation can hold (LF features each);
    // NSB: transposition sub-blocks (SBF features each) it can hold.  a.fw <= min(NLD*LF, NSB*SBF).
    constexpr int LF = 4 * VEC;              // features covered by one vector load of the wave
    constexpr int SBF = 16 * VEC;            // features per transposition sub-block
    constexpr int NT = NSB * VEC;            // 16-feature output tiles of the transposed product
    constexpr int STR = SBF + VEC;           // scratch row stride (elements): 16 bytes of padding
    constexpr bool HAS_C = (MODE == ROW_GRAD || MODE == ROW_APPLY);

    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, nw = blockDim.x >> 6;
    const int q = lane & 15, g = lane >> 4;
    const int K = a.K;
    const int64_t p = a.p;
    const int fw = a.fw;
    const int nld = (fw + LF - 1) / LF;                      // loads this launch really needs
    const int nsb = (fw + SBF - 1) / SBF;
    const int wrows = (nw - 1) * fw + nld * LF;              // rows of the LDS copy of M (zero beyond p)
    T *wl = (T *)smem_raw;
    T *zpart = wl + ((size_t)wrows * K + VEC - 1) / VEC * VEC;   // nw x 4 x 64 partial margins (16-byte aligned)
    T *zfull = zpart + (size_t)nw * 256 * (HAS_C ? 1 : 2);   // U of the block (modes with a transposed product)
    T *scr = zfull + 256 + (size_t)w * 16 * STR;             // wave-private transposition scratch

    {
        const T *M = (const T *)a.M;
        // batches of 8 independent loads per thread, so the copy costs one or two memory round trips
        const int total = wrows * K;
        for (int base = 0; base < total; base += 8 * (int)blockDim.x) {
            T tmp[8];
#pragma unroll
            for (int uu = 0; uu < 8; ++uu) {
                const int idx = base + uu * (int)blockDim.x + tid;
                const int f = idx / K, c = idx - f * K;
                tmp[uu] = (idx < total && f < p) ? M[(int64_t)f * a.ldm + c] : T(0);
            }
#pragma unroll
            for (int uu = 0; uu < 8; ++uu) {
                const int idx = base + uu * (int)blockDim.x + tid;
                if (idx < total) wl[idx] = tmp[uu];
            }
        }
    }
    __syncthreads();

    const T *X = (const T *)a.X;
    const int fs = w * fw;
    const int64_t fend = (fs + fw < p) ? (int64_t)(fs + fw) : p;   // features [fs, fend) belong to this wave
    const int qc = (q < K) ? q : K - 1;
    const bool cvalid = q < K;
    const int64_t nblk = (a.nrows + 15) / 16;

    // sample position -> data row of the lane's A-operand row of block rb
    auto block_row = [&](int64_t rb) -> int64_t {
        int64_t si = rb * 16 + q;
        if (si >= a.nrows) si = a.nrows - 1;
        return a.S ? (int64_t)a.S[si] : si;
    };
    auto load_block = [&](int64_t xr, pack(&x)[NLD]) {
        const T *xrow = X + xr * a.ldx;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            if (j < nld) {
                const int64_t f = fs + LF * j + VEC * g;
                if (f + VEC <= fend) {
                    x[j] = *(const pack *)(xrow + f);
                } else {
#pragma unroll
                    for (int m = 0; m < VEC; ++m) x[j].v[m] = (f + m < fend) ? xrow[f + m] : T(0);
                }
            }
        }
    };
    // accumulator elements (row groups) whose per-row work this wave does
    int vmask = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        if (nw == 1 || v % nw == w) vmask |= 1 << v;

    v4 G[HAS_C ? NT : 1];
#pragma unroll
    for (int t = 0; t < (HAS_C ? NT : 1); ++t) G[t] = v4{0, 0, 0, 0};
    double loss = 0.0;
    int hits = 0;

    int it = 0;
    pack xn[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) xn[j] = pack{};          // loads beyond the slice stay zero
    int64_t rb = blockIdx.x;
    if (rb < nblk) load_block(block_row(rb), xn);
    for (; rb < nblk; rb += gridDim.x) {
        pack xc[NLD];
#pragma unroll
        for (int j = 0; j < NLD; ++j) xc[j] = xn[j];
        // Small loads first (row index of the next block, labels / probabilities of this block), the X
        // prefetch after them: the memory counter retires in order, so the epilogue's wait for its inputs
        // then leaves the prefetch in flight.
        const int64_t rbn = rb + gridDim.x;
        const int64_t xr_next = (rbn < nblk) ? block_row(rbn) : 0;
        int lab_pre[4];
        T pin_pre[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            lab_pre[v] = 0;
            pin_pre[v] = T(0);
            if ((vmask >> v) & 1) {
                int64_t sv = rb * 16 + d_row<T>(g, v);
                if (sv >= a.nrows) sv = a.nrows - 1;
                if constexpr (MODE == ROW_APPLY) pin_pre[v] = ((const T *)a.Pin)[sv * a.KP + q];
                else if constexpr (MODE != ROW_PREP) lab_pre[v] = a.labels[a.S ? (int64_t)a.S[sv] : sv];
            }
        }
        if (rbn < nblk) load_block(xr_next, xn);

        // phase A: two accumulators break the dependent MFMA chain
        v4 z0 = v4{0, 0, 0, 0}, z1 = v4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            if (j < nld) {
#pragma unroll
                for (int m = 0; m < VEC; ++m) {
                    const int f = fs + LF * j + VEC * g + m;
                    const T bw = wl[f * K + qc];
                    const T b = cvalid ? bw : T(0);
                    if ((j * VEC + m) & 1) z1 = mfma16(xc[j].v[m], b, z1);
                    else z0 = mfma16(xc[j].v[m], b, z0);
                }
            }
            if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // keep the W operand reads from piling up
        }
        v4 z[1], u[1];
        z[0] = z0 + z1;
        u[0] = v4{0, 0, 0, 0};
        if (nw == 1) {
            row_epilogue<T, 1, MODE, true>(z, a, rb, lane, loss, hits, u, 15, lab_pre, pin_pre);
        } else {
            // partial margins -> LDS; wave w sums accumulator element v = w (, w+nw, ..) over the waves in a
            // fixed order and runs the per-row work for it, so the epilogue is done once per row block
            T *zp = zpart + (HAS_C ? 0 : (size_t)(it & 1) * nw * 256);
#pragma unroll
            for (int v = 0; v < 4; ++v) zp[(w * 4 + v) * 64 + lane] = z[0][v];
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if ((vmask >> v) & 1) {
                    T sacc = 0;
                    for (int ww = 0; ww < nw; ++ww) sacc += zp[(ww * 4 + v) * 64 + lane];
                    z[0][v] = sacc;
                }
            }
            if (vmask) row_epilogue<T, 1, MODE, true>(z, a, rb, lane, loss, hits, u, vmask, lab_pre, pin_pre);
            if constexpr (HAS_C) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if ((vmask >> v) & 1) zfull[v * 64 + lane] = u[0][v];
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 4; ++v) u[0][v] = zfull[v * 64 + lane];
            }
        }
        ++it;

        if constexpr (HAS_C) {
#pragma unroll
            for (int h = 0; h < NSB; ++h) {
                if (h < nsb) {
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        if (4 * h + jj < NLD) *(pack *)(scr + q * STR + LF * jj + VEC * g) = xc[4 * h + jj];
                        else *(pack *)(scr + q * STR + LF * jj + VEC * g) = pack{};
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const pack c = *(const pack *)(scr + d_row<T>(g, i) * STR + VEC * q);
#pragma unroll
                        for (int m = 0; m < VEC; ++m) G[h * VEC + m] = mfma16(c.v[m], u[0][i], G[h * VEC + m]);
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
    }

    if constexpr (HAS_C) {
        T *part = (T *)a.part + (int64_t)blockIdx.x * p * K;
#pragma unroll
        for (int h = 0; h < NSB; ++h)
#pragma unroll
            for (int m = 0; m < VEC; ++m)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int64_t f = fs + h * SBF + VEC * d_row<T>(g, v) + m;
                    if (h < nsb && f < fend && q < K) part[f * K + q] = G[h * VEC + m][v];
                }
    }
    // four partials per workgroup: wave w < 4 owns the rows of accumulator element w
    if (w < 4) {
        if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD) {
            for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
            if (lane == 0) a.loss_part[blockIdx.x * 4 + w] = loss;
            if (w == 0 && lane > 0 && lane < 4 && lane >= nw) a.loss_part[blockIdx.x * 4 + lane] = 0.0;
        } else if constexpr (MODE == ROW_PRED) {
            for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
            if (lane == 0) a.hit_part[blockIdx.x * 4 + w] = hits;
            if (w == 0 && lane > 0 && lane < 4 && lane >= nw) a.hit_part[blockIdx.x * 4 + lane] = 0;
        }
    }
}

constexpr int FUSED_MAX_FW = 128;    // features per wave the largest instantiation holds
constexpr int FUSED_MAX_WAVES = 8;   // 2 waves per SIMD: 256 registers each

// Split p features over nw waves of fw features each (fw a multiple of the vector width).
template <typename T> static void fused_shape(int64_t p, int *nw, int *fw)
{
    constexpr int VEC = 16 / sizeof(T);
    int n = (int)((p + FUSED_MAX_FW - 1) / FUSED_MAX_FW);
    if (n > 2) n = (n + 3) / 4 * 4;                 // same number of waves on each of the 4 SIMDs
    int f = (int)((p + n - 1) / n);
    f = (f + VEC - 1) / VEC * VEC;
    *nw = n;
    *fw = f;
}

template <typename T> static size_t fused_lds_bytes(int nw, int fw, int K, bool has_c)
{
    constexpr int VEC = 16 / sizeof(T);
    constexpr int LF = 4 * VEC, STR = 16 * VEC + VEC;
    const int nld = (fw + LF - 1) / LF;
    const size_t wrows = (size_t)(nw - 1) * fw + (size_t)nld * LF;
    size_t elems = (wrows * K + VEC - 1) / VEC * VEC + (size_t)nw * 256 * (has_c ? 1 : 2) + 256;
    if (has_c) elems += (size_t)nw * 16 * STR;
    return elems * sizeof(T);
}

template <typename T> static bool fused_ok(const RowsArgs &a)
{
    if (a.K > 16 || !vec_ok<T>(a.X, a.ldx)) return false;
    int nw, fw;
    fused_shape<T>(a.p, &nw, &fw);
    return nw <= FUSED_MAX_WAVES && fw <= FUSED_MAX_FW && fused_lds_bytes<T>(nw, fw, a.K, true) <= 160 * 1024;
}

// Can the one-pass kernel serve this shape?  (one 16-column class tile, 16-byte aligned rows, at most
// 8 waves of 128 features, LDS within the 160 KB of a gfx950 compute unit)
bool dense_fused_supported(int dtype, const RowsArgs &a)
{
    return dtype == SSN_F32 ? fused_ok<float>(a) : fused_ok<double>(a);
}

int dense_fused_grid(int dtype, const RowsArgs &a, int num_cus)
{
    int nw, fw;
    if (dtype == SSN_F32) fused_shape<float>(a.p, &nw, &fw);
    else fused_shape<double>(a.p, &nw, &fw);
    int per_cu = 8 / nw;                          // aim at 8 waves per compute unit
    if (per_cu < 1) per_cu = 1;
    const int64_t nblk = (a.nrows + 15) / 16;
    int64_t grid = (int64_t)num_cus * per_cu;
    if (grid > nblk) grid = nblk;
    if (grid < 1) grid = 1;
    return (int)grid;
}

template <typename T, int MODE, int NLD, int NSB>
static hipError_t fused_launch_inst(const RowsArgs &a, int grid, int nw, size_t lds, hipStream_t st)
{
    auto kern = dense_fused_kernel<T, MODE, NLD, NSB>;
    static size_t lds_allowed = 48 * 1024;          // raise the dynamic LDS limit once per instantiation
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_allowed = 160 * 1024;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * nw), lds, st, a);
    return hipGetLastError();
}

template <typename T, int MODE> static hipError_t fused_launch_mode(RowsArgs a, int grid, hipStream_t st)
{
    constexpr int VEC = 16 / sizeof(T);
    constexpr int LF = 4 * VEC, SBF = 16 * VEC;
    int nw, fw;
    fused_shape<T>(a.p, &nw, &fw);
    a.fw = fw;
    constexpr bool has_c = (MODE == ROW_GRAD || MODE == ROW_APPLY);
    const size_t lds = fused_lds_bytes<T>(nw, fw, a.K, has_c);
    // three register footprints: <= 64, <= 104 (f64) / 112 (f32), <= 128 features per wave
    constexpr int MID_LD = (sizeof(T) == 8) ? 13 : 7;
    if (fw <= 64) return fused_launch_inst<T, MODE, 64 / LF, 64 / SBF>(a, grid, nw, lds, st);
    if (fw <= MID_LD * LF) return fused_launch_inst<T, MODE, MID_LD, 128 / SBF>(a, grid, nw, lds, st);
    return fused_launch_inst<T, MODE, 128 / LF, 128 / SBF>(a, grid, nw, lds, st);
}

template <typename T> static hipError_t fused_dispatch(const RowsArgs &a, int grid, hipStream_t st)
{
    switch (a.mode) {
    case ROW_OBJ: return fused_launch_mode<T, ROW_OBJ>(a, grid, st);
    case ROW_GRAD: return fused_launch_mode<T, ROW_GRAD>(a, grid, st);
    case ROW_PREP: return fused_launch_mode<T, ROW_PREP>(a, grid, st);
    case ROW_APPLY: return fused_launch_mode<T, ROW_APPLY>(a, grid, st);
    case ROW_PRED: return fused_launch_mode<T, ROW_PRED>(a, grid, st);
    default: return hipErrorInvalidValue;
    }
}

// Launch the one-pass kernel on `grid` workgroups; ROW_GRAD / ROW_APPLY leave `grid` partials in a.part,
// ROW_OBJ / ROW_GRAD `grid` loss partials, ROW_PRED `grid` hit partials.
hipError_t launch_dense_fused(int dtype, const RowsArgs &a, int grid, hipStream_t st)
{
    return dtype == SSN_F32 ? fused_dispatch<float>(a, grid, st) : fused_dispatch<double>(a, grid, st);
}

}  // namespace ssn
