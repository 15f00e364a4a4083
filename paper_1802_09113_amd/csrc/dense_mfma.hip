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
#include "ssn_math.h"

#include <cstdlib>
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

// TIGHT: the caller has no registers to spare (see exp_nonpos)
template <bool TIGHT> __device__ __forceinline__ float t_exp(float x) { return expf(x); }
template <bool TIGHT> __device__ __forceinline__ double t_exp(double x) { return exp_nonpos(x, TIGHT ? opaque_zero() : 0.0); }
__device__ __forceinline__ float t_log(float x) { return logf(x); }
__device__ __forceinline__ double t_log(double x) { return log_ge1(x); }

// Reductions over the 16 lanes that hold the 16 class columns of one row: four rotate-and-combine steps
// inside the row (DPP row_ror 8, 4, 2, 1 -- register-to-register, no trip through the LDS crossbar),
// after which every lane of the row holds the result.
template <int ROT> __device__ __forceinline__ int dpp_ror(int x)
{
    return __builtin_amdgcn_update_dpp(x, x, 0x120 + ROT, 0xF, 0xF, false);
}
template <int ROT> __device__ __forceinline__ float row_ror(float x) { return __int_as_float(dpp_ror<ROT>(__float_as_int(x))); }
template <int ROT> __device__ __forceinline__ double row_ror(double x)
{
    return __hiloint2double(dpp_ror<ROT>(__double2hiint(x)), dpp_ror<ROT>(__double2loint(x)));
}
template <int ROT> __device__ __forceinline__ int row_ror(int x) { return dpp_ror<ROT>(x); }
template <typename T> __device__ __forceinline__ T row16_sum(T x)
{
    x += row_ror<8>(x);
    x += row_ror<4>(x);
    x += row_ror<2>(x);
    x += row_ror<1>(x);
    return x;
}
template <typename T> __device__ __forceinline__ T row16_max(T x)
{
    x = fmax(x, row_ror<8>(x));
    x = fmax(x, row_ror<4>(x));
    x = fmax(x, row_ror<2>(x));
    x = fmax(x, row_ror<1>(x));
    return x;
}
__device__ __forceinline__ int row16_min(int x)
{
    x = min(x, row_ror<8>(x));
    x = min(x, row_ror<4>(x));
    x = min(x, row_ror<2>(x));
    x = min(x, row_ror<1>(x));
    return x;
}

// 1 / a for a in [1, 17]: hardware estimate plus two Newton steps (about one ulp), a fraction of the
// instructions of an IEEE division
__device__ __forceinline__ double fast_rcp(double a)
{
    double x = __builtin_amdgcn_rcp(a);
    x = fma(fma(-a, x, 1.0), x, x);
    x = fma(fma(-a, x, 1.0), x, x);
    return x;
}
__device__ __forceinline__ float fast_rcp(float a)
{
    float x = __builtin_amdgcn_rcpf(a);
    x = fmaf(fmaf(-a, x, 1.0f), x, x);
    return x;
}

// ---------------------------------------------------------------------------------------------
// Per-row work on ONE accumulator element of a 16-row block (K <= 16): the 16 lanes of a row group hold the
// 16 class columns of sample row sv.  lab / pin are that row's label and this lane's probability,
// loaded by the caller.  Returns U (ROW_GRAD: eq. (6) residual p - y; ROW_APPLY: eq. (12)).
template <typename T, int MODE, bool TIGHT = false>
__device__ __forceinline__ T slot_epilogue(T z, const RowsArgs &a, int64_t sv, int q, int lab, T pin, double &loss,
                                           double &lprod, int &hits)
{
    const int K = a.K;
    const bool valid = sv < a.nrows;
    const bool cv = q < K;
    const T NEG = -std::numeric_limits<T>::infinity();
    if constexpr (MODE == ROW_APPLY) {
        const T t = row16_sum(pin * z);                    // pin is zero in padded columns
        const T u = valid ? (pin * z - pin * t) : T(0);
        // z_i . u_i of the row: summed over the sample it is V^T (X_S^T U), the curvature term CG needs
        const T zu = row16_sum(z * u);
        if (valid && q == 0) loss += (double)zu;
        return u;
    }
    if constexpr (MODE == ROW_PRED) {
        const T zmax = row16_max(cv ? z : NEG);
        const int cand = row16_min((cv && z == zmax) ? q : 0x7fffffff);
        const int pr = (T(0) > zmax) ? K : cand;           // the reference class wins only strictly
        if (valid && q == 0) {
            if (a.pred) a.pred[sv] = pr;
            hits += (pr == lab);
        }
        return T(0);
    }
    // eqs. (8), (9).  With K < 16 the lane of column K is free: it plays the reference class (margin 0), so
    // M = max{0, z} is one row maximum and alpha = e^{-M} + sum_c e^{z_c - M} one row sum of one
    // exponential per lane.
    const bool ref_lane = K < 16;
    const T zz = (q == K) ? T(0) : z;
    const bool ce = ref_lane ? (q <= K) : cv;
    const T zmax = row16_max(ce ? zz : NEG);
    const T Mx = ref_lane ? zmax : fmax(T(0), zmax);
    const T e = ce ? t_exp<TIGHT>(zz - Mx) : T(0);
    T alpha = row16_sum(e);
    if (!ref_lane) alpha += t_exp<TIGHT>(-Mx);
    const T inv = fast_rcp(alpha);
    if constexpr (MODE == ROW_PREP) {
        ((T *)a.UP)[sv * a.KP + q] = (valid && cv) ? e * inv : T(0);
        return T(0);
    }
    // margin of the label's class, read from the lane that holds it (0 for the reference class)
    const T zl = __shfl(z, (threadIdx.x & 48) | (lab & 15));
    const T lin = (lab < K) ? zl : T(0);
    // eqs. (14)-(17): the row adds M + log(alpha) - z_label.  The logarithms are taken of a running product
    // of the alphas (each in [1, C]) instead of one by one; the product is folded into the sum before it
    // can overflow, and once more at the end of the kernel.
    if (valid && q == 0) {
        loss += (double)Mx - (double)lin;
        lprod *= (double)alpha;
    }
    if (lprod > 1e250) {
        loss += log(lprod);
        lprod = 1.0;
    }
    if constexpr (MODE == ROW_GRAD) return (valid && cv) ? (e * inv - ((q == lab) ? T(1) : T(0))) : T(0);
    return T(0);
}

// ---------------------------------------------------------------------------------------------
// Two accumulator elements at once for K <= 7 (ROW_OBJ / ROW_GRAD): with at most seven weight columns plus the
// reference class a row needs 8 of its 16 lanes, so lanes 8..15 take the row of a second accumulator element
// (DPP rotation by 8 inside the 16-lane row) and the exponentials, reciprocals and reductions of both rows cost
// one pass.  In the kernels whose workgroup is a single wave this per-row work is about half of the time.
template <int CTRL> __device__ __forceinline__ int dpp_mov(int x)
{
    return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_val(float x) { return __int_as_float(dpp_mov<CTRL>(__float_as_int(x))); }
template <int CTRL> __device__ __forceinline__ double dpp_val(double x)
{
    return __hiloint2double(dpp_mov<CTRL>(__double2hiint(x)), dpp_mov<CTRL>(__double2loint(x)));
}
// reductions over the 8 lanes of a half row: neighbours, pairs (quad permutations 1032 and 2301), then the
// mirror image inside the half row; every lane of the half row ends with the result
template <typename T> __device__ __forceinline__ T half8_sum(T x)
{
    x += dpp_val<0xB1>(x);
    x += dpp_val<0x4E>(x);
    x += dpp_val<0x141>(x);
    return x;
}
template <typename T> __device__ __forceinline__ T half8_max(T x)
{
    x = fmax(x, dpp_val<0xB1>(x));
    x = fmax(x, dpp_val<0x4E>(x));
    x = fmax(x, dpp_val<0x141>(x));
    return x;
}
// za / zb: the lane's margins of elements a and b (class q of rows sva / svb, labels laba / labb); ub receives
// element b's result, the return value is element a's (both zero in lanes 8..15, which hold no class of theirs)
template <typename T, int MODE>
__device__ __forceinline__ T slot_epilogue_pair(T za, T zb, T &ub, const RowsArgs &a, int64_t sva, int64_t svb, int q, int laba,
                                                int labb, double &loss, double &lprod)
{
    static_assert(MODE == ROW_OBJ || MODE == ROW_GRAD, "paired per-row work: loss modes only");
    const int K = a.K;                                   // <= 7: lane K of the half row is free for the reference class
    const bool hi = q >= 8;
    const int qh = q & 7;
    const T zb_up = dpp_val<0x128>(zb);                  // rotation by 8 inside the row: lane q takes lane q +- 8
    const T z = hi ? zb_up : za;
    const int64_t sv = hi ? svb : sva;
    const int lab = hi ? labb : laba;
    const bool valid = sv < a.nrows;
    const bool cv = qh < K;
    const T NEG = -std::numeric_limits<T>::infinity();
    // eqs. (8), (9) as in slot_epilogue, on half rows
    const T zz = (qh == K) ? T(0) : z;
    const bool ce = qh <= K;
    const T Mx = half8_max(ce ? zz : NEG);
    const T e = ce ? t_exp<false>(zz - Mx) : T(0);
    const T alpha = half8_sum(e);
    const T inv = fast_rcp(alpha);
    const T zl = __shfl(z, (threadIdx.x & 56) | (lab & 7));          // same row group, same half row
    const T lin = (lab < K) ? zl : T(0);
    if (valid && qh == 0) {
        loss += (double)Mx - (double)lin;
        lprod *= (double)alpha;
    }
    if (lprod > 1e250) {
        loss += log(lprod);
        lprod = 1.0;
    }
    if constexpr (MODE == ROW_GRAD) {
        const T u = (valid && cv) ? (e * inv - ((qh == lab) ? T(1) : T(0))) : T(0);
        const T u_dn = dpp_val<0x128>(u);
        ub = hi ? T(0) : u_dn;
        return hi ? T(0) : u;
    }
    ub = T(0);
    return T(0);
}

// Per-row work on a 16-row block of margins held in MFMA accumulator layout:
// acc[nb][v] = z(row d_row<T>(lane/16, v), class 16*nb + lane%16).  With one class tile (K <= 16) the
// modes that exponentiate go through slot_epilogue, element by element.
template <typename T, int NB, int MODE>
__device__ __forceinline__ void row_epilogue(const typename V4<T>::type (&acc)[NB], const RowsArgs &a,
                                             int64_t rb, int lane, double &loss, double &lprod, int &hits)
{
    const int q = lane & 15, g = lane >> 4;
    const int K = a.K;
    const T NEG = -std::numeric_limits<T>::infinity();
    if constexpr (MODE == ROW_MARGIN) {                  // the margins of both operands, 2K values per row
        T *Z = (T *)a.UP;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t sv = rb * 16 + d_row<T>(g, v);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                if (sv < a.nrows && nb * 16 + q < 2 * K) Z[sv * a.KP + nb * 16 + q] = acc[nb][v];
        }
        return;
    }
    if constexpr (NB == 1 && (MODE == ROW_OBJ || MODE == ROW_GRAD)) {
        if (K <= 7) {                                    // two accumulator elements per pass
#pragma unroll
            for (int v = 0; v < 4; v += 2) {
                const int64_t sva = rb * 16 + d_row<T>(g, v), svb = rb * 16 + d_row<T>(g, v + 1);
                const int64_t ca = sva < a.nrows ? sva : a.nrows - 1, cb = svb < a.nrows ? svb : a.nrows - 1;
                const int laba = a.labels[a.S ? a.S[ca] : ca], labb = a.labels[a.S ? a.S[cb] : cb];
                T ub;
                const T ua = slot_epilogue_pair<T, MODE>(acc[0][v], acc[0][v + 1], ub, a, sva, svb, q, laba, labb, loss, lprod);
                if constexpr (MODE == ROW_GRAD) {
                    ((T *)a.UP)[sva * a.KP + q] = ua;
                    ((T *)a.UP)[svb * a.KP + q] = ub;
                }
            }
            return;
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int64_t sv = rb * 16 + d_row<T>(g, v);
        const bool valid = sv < a.nrows;
        const int64_t svc = valid ? sv : a.nrows - 1;
        if constexpr (NB == 1 && (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_PREP)) {
            int lab = 0;
            if constexpr (MODE != ROW_PREP) lab = a.labels[a.S ? a.S[svc] : svc];
            const T u = slot_epilogue<T, MODE>(acc[0][v], a, sv, q, lab, T(0), loss, lprod, hits);
            if constexpr (MODE == ROW_GRAD) ((T *)a.UP)[sv * a.KP + q] = u;
            continue;
        }
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
            const int lab = a.labels[a.S ? a.S[svc] : svc];
            int cand = 0x7fffffff;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                if (cv[nb] && z[nb] == zmax) cand = min(cand, nb * 16 + q);
            cand = row16_min(cand);
            const int pr = (T(0) > zmax) ? K : cand;     // the reference class wins only strictly
            if (valid && q == 0) {
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
                pin[nb] = Pin[svc * a.KP + nb * 16 + q];      // zero in padded columns
                t += pin[nb] * z[nb];
            }
            t = row16_sum(t);
            T *U = (T *)a.UP;
            T zu = 0;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const T u = valid ? (pin[nb] * z[nb] - pin[nb] * t) : T(0);
                zu += z[nb] * u;
                U[sv * a.KP + nb * 16 + q] = u;
            }
            // z_i . u_i of the row: summed over the sample it is V^T (X_S^T U), the curvature term CG needs
            zu = row16_sum(zu);
            if (valid && q == 0) loss += (double)zu;
            continue;
        }
        // eq. (8), (9): M = max{0, z}, alpha = e^{-M} + sum_c e^{z_c - M}
        const T Mx = fmax(T(0), zmax);
        T e[NB];
        T se = 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            e[nb] = cv[nb] ? t_exp<false>(z[nb] - Mx) : T(0);
            se += e[nb];
        }
        se = row16_sum(se);
        const T alpha = t_exp<false>(-Mx) + se;
        if constexpr (MODE == ROW_PREP) {
            T *P = (T *)a.UP;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                P[sv * a.KP + nb * 16 + q] = valid ? e[nb] / alpha : T(0);
            continue;
        }
        // ROW_OBJ / ROW_GRAD: eqs. (14)-(17)
        const int lab = a.labels[a.S ? a.S[svc] : svc];
        T lin = 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            lin += (cv[nb] && (nb * 16 + q) == lab) ? z[nb] : T(0);
        lin = row16_sum(lin);
        if (valid && q == 0) loss += (double)Mx + (double)t_log(alpha) - (double)lin;
        if constexpr (MODE == ROW_GRAD) {
            T *U = (T *)a.UP;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const T ind = ((nb * 16 + q) == lab) ? T(1) : T(0);
                const T u = (valid && cv[nb]) ? (e[nb] / alpha - ind) : T(0);
                U[sv * a.KP + nb * 16 + q] = u;
            }
        }
    }
}

// One wave per 16-row block; grid-stride over row blocks.  UP / Pin have ceil(nrows/16)*16 rows.
//
// SPLIT: for a few thousand rows there are too few row blocks to fill the chip with one wave each, and a
// wave that walks all p features alone is a long chain of dependent loads.  Then a whole workgroup (8 or
// 16 waves; 4 on full passes over matrices of 2048 features and more) shares one row block: the waves take
// the feature groups in turn, their partial margins are added through LDS in wave order, and wave 0 does the
// per-row work.
//
// PAIR: two row blocks per trip share every load of W, which otherwise costs the L1 as many bytes as X
// itself (wide matrices; for narrow ones the per-row work dominates and more, smaller trips are better).
// (A class-major copy of M, one vector load per lane for the W operands of consecutive features, was
// tried: its loads touch 16 cache lines per instruction instead of 4-8 and the kernel got 30 % slower.)
template <typename T, int NB, int VEC, int MODE, bool SPLIT, bool PAIR>
__global__ __launch_bounds__(SPLIT ? 1024 : 64 * ROWS_WAVES_PER_BLOCK) void dense_rows_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    typedef Pack<T, VEC> pack;
    extern __shared__ __align__(16) unsigned char rows_smem[];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const int nsw = blockDim.x >> 6;                  // SPLIT: waves sharing the row block
    const int q = lane & 15, g = lane >> 4;
    const int64_t nwaves = SPLIT ? (int64_t)gridDim.x : (int64_t)gridDim.x * ROWS_WAVES_PER_BLOCK;
    const int64_t wave = SPLIT ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * ROWS_WAVES_PER_BLOCK + wib;
    const T *X = (const T *)a.X;
    const T *M = (const T *)a.M;
    const int K = a.K;
    const int64_t p = a.p, ldm = a.ldm;

    // this lane's column of the right operand; ROW_MARGIN: columns K..2K-1 are the columns of the second operand
    bool cval[NB];
    const T *mcol[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int c = nb * 16 + q;
        if constexpr (MODE == ROW_MARGIN) {
            cval[nb] = c < 2 * K;
            mcol[nb] = (c >= K && cval[nb]) ? (const T *)a.M2 + (c - K) : M + (c < K ? c : K - 1);
        } else {
            cval[nb] = c < K;
            mcol[nb] = M + (cval[nb] ? c : K - 1);
        }
    }

    double loss = 0.0, lprod = 1.0;         // sum of the row terms without log(alpha); product of the alphas
    int hits = 0;
    const int64_t nblk = (a.nrows + 15) / 16;
    constexpr int STEP = 4 * VEC;     // features consumed per vector load (4 k-groups of VEC)
    // Loads in flight per trip.  A 16-wave workgroup leaves 128 registers per lane; with four vector loads and
    // their W operands in flight some variants spilled, and a kernel that uses scratch memory at all pays
    // ~14 us per launch on this machine, more than a whole sampled product: those variants take fewer.
    constexpr bool EXPS = (MODE == ROW_OBJ || MODE == ROW_GRAD);      // fp64 exp / log routines in the epilogue
    constexpr int UNR = !SPLIT ? 4 : (sizeof(T) == 8 && NB == 2 && (EXPS || MODE == ROW_PREP)) ? 1 : (sizeof(T) == 4 || NB == 2 || EXPS) ? 2 : 4;

    constexpr int RB = PAIR ? 2 : 1;
    for (int64_t rb0 = wave * RB; rb0 < nblk; rb0 += nwaves * RB) {
        const T *xrow[RB];
        v4 acc[RB][NB];
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            int64_t si = (rb0 + k) * 16 + q;
            if (si >= a.nrows) si = a.nrows - 1;      // clamped rows are masked in the epilogue
            const int64_t xr = a.S ? a.S[si] : si;
            xrow[k] = X + xr * a.ldx;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[k][nb] = v4{0, 0, 0, 0};
        }

        int64_t f0 = SPLIT ? (int64_t)wib * (STEP * UNR) : 0;
        const int64_t fstride = SPLIT ? (int64_t)nsw * (STEP * UNR) : STEP * UNR;
        for (; f0 + STEP * UNR <= p; f0 += fstride) {
            pack xv[RB][UNR];
            T wv[UNR][VEC][NB];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int64_t f = f0 + u * STEP + VEC * g;
#pragma unroll
                for (int k = 0; k < RB; ++k) xv[k][u] = *(const pack *)(xrow[k] + f);
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
                    for (int nb = 0; nb < NB; ++nb) {
                        const T w = cval[nb] ? wv[u][m][nb] : T(0);
#pragma unroll
                        for (int k = 0; k < RB; ++k) acc[k][nb] = mfma16(xv[k][u].v[m], w, acc[k][nb]);
                    }
        }
        f0 = p / (STEP * UNR) * (STEP * UNR);
        if (SPLIT && wib != 0) f0 = p;                 // the tail belongs to wave 0
        for (; f0 < p; f0 += STEP) {                   // guarded tail
            const int64_t f = f0 + VEC * g;
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const bool ok = (f + m) < p;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const T w = (ok && cval[nb]) ? mcol[nb][(f + m) * ldm] : T(0);
#pragma unroll
                    for (int k = 0; k < RB; ++k) {
                        const T x = ok ? xrow[k][f + m] : T(0);
                        acc[k][nb] = mfma16(x, w, acc[k][nb]);
                    }
                }
            }
        }
        if constexpr (SPLIT) {
            const int64_t rb = rb0;
            T *zs = (T *)rows_smem;                    // nsw x NB x 4 x 64
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 4; ++v) zs[((wib * NB + nb) * 4 + v) * 64 + lane] = acc[0][nb][v];
            __syncthreads();
            if (wib == 0) {
                for (int ww = 1; ww < nsw; ++ww)       // fixed order
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[0][nb][v] += zs[((ww * NB + nb) * 4 + v) * 64 + lane];
                row_epilogue<T, NB, MODE>(acc[0], a, rb, lane, loss, lprod, hits);
            }
            __syncthreads();
        } else {
#pragma unroll
            for (int k = 0; k < RB; ++k)
                if (rb0 + k < nblk) row_epilogue<T, NB, MODE>(acc[k], a, rb0 + k, lane, loss, lprod, hits);
        }
    }

    // one partial per wave; SPLIT: the block's four partial slots are wave 0's sum and three zeros
    if (SPLIT && wib != 0) return;
    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
        if constexpr (MODE != ROW_APPLY) loss += log(lprod);
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
        if constexpr (SPLIT) {
            if (lane < ROWS_WAVES_PER_BLOCK) a.loss_part[wave * ROWS_WAVES_PER_BLOCK + lane] = (lane == 0) ? loss : 0.0;
        } else {
            if (lane == 0) a.loss_part[wave] = loss;
        }
    } else if constexpr (MODE == ROW_PRED) {
        for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
        if constexpr (SPLIT) {
            if (lane < ROWS_WAVES_PER_BLOCK) a.hit_part[wave * ROWS_WAVES_PER_BLOCK + lane] = (lane == 0) ? hits : 0;
        } else {
            if (lane == 0) a.hit_part[wave] = hits;
        }
    }
}

// part[chunk] (p x K) = sum over the chunk's rows of x_row^T u_row.
// Block = 4 waves, each wave owns 64 consecutive features; blockIdx.y = row chunk.
// A vector load of VEC consecutive features per lane feeds VEC MFMAs whose output rows are the
// features {base + VEC*i + m : i = 0..15}.
// FROMZ (one class tile): the rows of U are not read but formed here from the partial margins of a.nslices feature
// slices and the probabilities, eq. (12): the 16 lanes of a row group hold the 16 class columns of a row, as in the
// per-row work of the rows kernels.  Every feature tile's workgroup forms the same U (a few loads and a row
// reduction per four rows); the workgroup of the first tile also leaves the chunk's sum of z_i . u_i.
template <typename T, int NB, int VEC, bool FROMZ = false>
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
    double zu_sum = 0.0;
    // FROMZ: u of sample row sc, class q, from the row's margin z and probability pin (all 64 lanes take part: the
    // row sums are DPP rotations inside the row group)
    constexpr int MAXS = 4;                           // feature slices at most (the launcher's plan keeps to it)
    auto load_z = [&](int64_t sc, T (&zs)[MAXS], T &pin) {
        const T *zp = (const T *)a.Zpart + sc * 16 + q;
#pragma unroll
        for (int s = 0; s < MAXS; ++s) zs[s] = zp[(int64_t)(s < a.nslices ? s : 0) * a.zrows * 16];
        pin = ((const T *)a.Pin)[sc * a.KP + q];      // zero in padded columns
    };
    auto form_u = [&](const T (&zs)[MAXS], T pin, bool rv) -> T {
        T z = zs[0];
#pragma unroll
        for (int s = 1; s < MAXS; ++s) z += (s < a.nslices) ? zs[s] : T(0);      // slices in a fixed order
        const T t = row16_sum(pin * z);
        const T u = rv ? (pin * z - pin * t) : T(0);
        const T zu = row16_sum(z * u);
        if (q == 0) zu_sum += (double)zu;
        return u;
    };

    v4 acc[NL * VEC][NB];
#pragma unroll
    for (int t = 0; t < NL * VEC; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = v4{0, 0, 0, 0};

    // main loop: 16 rows (four MFMA contraction steps) per trip, every load of the trip issued before its
    // first MFMA; the guarded loop below takes the rest
    constexpr int RU = 4;
    int64_t r0 = r_begin;
    if (full) {
        for (; r0 + 4 * RU <= r_end; r0 += 4 * RU) {
            pack xv[RU][NL];
            T ub[RU][NB];
            T zsl[FROMZ ? RU : 1][MAXS], pinv[FROMZ ? RU : 1];
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int64_t sc = r0 + 4 * u + g;
                const int64_t xr = a.S ? (int64_t)a.S[sc] : sc;
                const T *xrow = X + xr * a.ldx + f0 + VEC * q;
#pragma unroll
                for (int ld = 0; ld < NL; ++ld) xv[u][ld] = *(const pack *)(xrow + ld * 16 * VEC);
                if constexpr (FROMZ) {
                    load_z(sc, zsl[u], pinv[u]);      // every load of the trip is issued before the first row sum
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) ub[u][nb] = U[sc * a.KP + nb * 16 + q];
                }
            }
            if constexpr (FROMZ) {
#pragma unroll
                for (int u = 0; u < RU; ++u) ub[u][0] = form_u(zsl[u], pinv[u], true);
            }
#pragma unroll
            for (int u = 0; u < RU; ++u)
#pragma unroll
                for (int ld = 0; ld < NL; ++ld)
#pragma unroll
                    for (int m = 0; m < VEC; ++m)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[ld * VEC + m][nb] = mfma16(xv[u][ld].v[m], ub[u][nb], acc[ld * VEC + m][nb]);
        }
    }
    for (; r0 < r_end; r0 += 4) {
        const int64_t si = r0 + g;
        const bool rv = si < r_end;
        const int64_t sc = rv ? si : r_begin;
        const int64_t xr = a.S ? a.S[sc] : sc;
        const T *xrow = X + xr * a.ldx + f0;
        T ub[NB];
        if constexpr (FROMZ) {
            T zs1[MAXS], pin1;
            load_z(sc, zs1, pin1);
            ub[0] = form_u(zs1, pin1, rv);
        } else {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const T u = U[sc * a.KP + nb * 16 + q];
                ub[nb] = rv ? u : T(0);
            }
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

    if constexpr (FROMZ) {
        if (blockIdx.x == 0 && wib == 0) {           // one sum of z_i . u_i per chunk, from the first feature tile's wave
            for (int off = 32; off > 0; off >>= 1) zu_sum += __shfl_xor(zu_sum, off);
            if (lane == 0) a.zu_part[chunk] = zu_sum;
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

// fp32 rows that are only 8-byte aligned (e.g. 54 features): two-element vector loads
static bool half_vec_ok(int dtype_size, const void *X, int64_t ldx)
{
    return dtype_size == 4 && ((uintptr_t)X % 8 == 0) && (ldx % 2 == 0);
}

template <typename T> static bool vec_ok(const void *X, int64_t ldx)
{
    constexpr int VEC = 16 / sizeof(T);
    return ((uintptr_t)X % 16 == 0) && (ldx % VEC == 0);
}

// Partial margins of feature slices, for products on a sample of a few thousand rows of a wide matrix: such a sample
// has fewer 16-row blocks than the chip has compute units, so a workgroup per row block leaves a third of them idle
// and each workgroup walks all p features.  Here a workgroup of eight waves takes one (row block, feature slice)
// pair; its waves take the slice's feature groups in turn and add their partial margins through LDS in wave order;
// the slices' partial margins Zpart[s][row][16] are added up, and eq. (12) applied, by the transposed-product kernel
// that follows (dense_xtu_kernel with FROMZ).
template <typename T, int VEC>
__global__ __launch_bounds__(512) void dense_zpart_kernel(RowsArgs a, T *Zpart, int nslices, int64_t fper)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    typedef Pack<T, VEC> pack;
    __shared__ T zs[8 * 256];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6, nsw = blockDim.x >> 6;
    const int q = lane & 15, g = lane >> 4;
    const int64_t rb = blockIdx.x / nslices;
    const int sl = blockIdx.x - (int)rb * nslices;
    const int64_t zrows = (a.nrows + 15) / 16 * 16;
    const T *X = (const T *)a.X;
    const int K = a.K;
    const int64_t p = a.p, ldm = a.ldm;
    const int64_t fbeg = (int64_t)sl * fper, fend = (fbeg + fper < p) ? fbeg + fper : p;
    const bool cval = q < K;
    const T *mcol = (const T *)a.M + (cval ? q : K - 1);
    int64_t si = rb * 16 + q;
    if (si >= a.nrows) si = a.nrows - 1;              // rows beyond the sample: computed, never used
    const T *xrow = X + (a.S ? (int64_t)a.S[si] : si) * a.ldx;
    constexpr int STEP = 4 * VEC, UNR = 4;
    v4 acc = v4{0, 0, 0, 0};
    int64_t f0 = fbeg + (int64_t)wib * (STEP * UNR);
    // the loads of the wave's next feature group are issued before the matrix instructions of the current one: a
    // wave has only a handful of groups, and waiting out a trip to memory between each two was most of its time
    auto fetch = [&](int64_t at, pack (&xv)[UNR], T (&wv)[UNR][VEC]) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t f = at + u * STEP + VEC * g;
            xv[u] = *(const pack *)(xrow + f);
#pragma unroll
            for (int m = 0; m < VEC; ++m) wv[u][m] = mcol[(f + m) * ldm];
        }
    };
    auto multiply = [&](const pack (&xv)[UNR], const T (&wv)[UNR][VEC]) {
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int m = 0; m < VEC; ++m) acc = mfma16(xv[u].v[m], cval ? wv[u][m] : T(0), acc);
    };
    const int64_t stride = (int64_t)nsw * (STEP * UNR);
    pack xa[UNR], xb[UNR];
    T wa[UNR][VEC], wb[UNR][VEC];
    bool have = f0 + STEP * UNR <= fend;
    if (have) fetch(f0, xa, wa);
    while (have) {
        const bool more = f0 + stride + STEP * UNR <= fend;
        if (more) fetch(f0 + stride, xb, wb);
        multiply(xa, wa);
        if (!more) break;
        const bool again = f0 + 2 * stride + STEP * UNR <= fend;
        if (again) fetch(f0 + 2 * stride, xa, wa);
        multiply(xb, wb);
        have = again;
        f0 += 2 * stride;
    }
    if (wib == 0) {                                   // the slice's last, incomplete group of features
        for (f0 = fbeg + (fend - fbeg) / (STEP * UNR) * (STEP * UNR); f0 < fend; f0 += STEP) {
            const int64_t f = f0 + VEC * g;
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const bool ok = (f + m) < fend;
                const T w = (ok && cval) ? mcol[(f + m) * ldm] : T(0);
                const T x = ok ? xrow[f + m] : T(0);
                acc = mfma16(x, w, acc);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) zs[(wib * 4 + v) * 64 + lane] = acc[v];
    __syncthreads();
    if (wib == 0) {
        for (int ww = 1; ww < nsw; ++ww)              // fixed order
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] += zs[(ww * 4 + v) * 64 + lane];
        T *zp = Zpart + ((int64_t)sl * zrows + rb * 16) * 16;
#pragma unroll
        for (int v = 0; v < 4; ++v) zp[d_row<T>(g, v) * 16 + q] = acc[v];
    }
}

hipError_t launch_dense_zpart(int dtype, const RowsArgs &a, void *Zpart, int nslices, int64_t fper, hipStream_t st)
{
    if (a.K > 16 || nslices < 1 || fper < 1) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)(((a.nrows + 15) / 16) * nslices);
    if (dtype == SSN_F32) {
        if (!vec_ok<float>(a.X, a.ldx) || fper % 64) return hipErrorInvalidValue;
        hipLaunchKernelGGL((dense_zpart_kernel<float, 4>), dim3(grid), dim3(512), 0, st, a, (float *)Zpart, nslices, fper);
    } else {
        if (!vec_ok<double>(a.X, a.ldx) || fper % 32) return hipErrorInvalidValue;
        hipLaunchKernelGGL((dense_zpart_kernel<double, 2>), dim3(grid), dim3(512), 0, st, a, (double *)Zpart, nslices, fper);
    }
    return hipGetLastError();
}

// Workgroups and waves per workgroup of the wave-per-row-block kernel: *split_waves == 0 is the plain
// form (4 waves, one row block each); otherwise each workgroup of *split_waves waves shares a row block.
void dense_rows_plan(int dtype, int64_t nrows, int64_t p, int K, int num_cus, int *blocks, int *split_waves)
{
    const int64_t nblk = (nrows + 15) / 16;
    const size_t es = dtype == SSN_F32 ? 4 : 8;
    const int nb = (K + 15) / 16;
    *split_waves = 0;
    *blocks = rows_grid_blocks(nrows, num_cus);
    if (nblk <= (int64_t)num_cus * 2 && p >= 512) {
        int w = p >= 2048 ? 16 : 8;
        if ((size_t)w * nb * 256 * es > 32768) w = 8;
        *split_waves = w;
        *blocks = (int)(nblk < 1 ? 1 : nblk);
    } else if (p >= 2048) {
        // all rows of a wide matrix: a wave that streams a whole row block alone keeps too little in flight; four
        // waves per block do better (50000 x 3072: fp64 objective 303 -> 280 us, fp32 180 -> 150 us; at 784
        // features the plain form wins)
        *split_waves = 4;
        const int64_t cap = (int64_t)num_cus * 16;           // beyond that the workgroups stride over the row blocks
        *blocks = (int)(nblk < cap ? nblk : cap);
    }
}

template <typename T, int MODE>
static hipError_t rows_dispatch_mode(const RowsArgs &a, int blocks, int split_waves, hipStream_t st)
{
    constexpr int VEC = 16 / sizeof(T);
    const int nb = ((MODE == ROW_MARGIN ? 2 * a.K : a.K) + 15) / 16;
    const bool v = vec_ok<T>(a.X, a.ldx);
    if (nb != 1 && nb != 2) return hipErrorInvalidValue;
    if (split_waves > 0 && v) {
        dim3 grid(blocks), block(64 * split_waves);
        const size_t lds = (size_t)split_waves * nb * 256 * sizeof(T);
        if (nb == 1) hipLaunchKernelGGL((dense_rows_kernel<T, 1, VEC, MODE, true, false>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((dense_rows_kernel<T, 2, VEC, MODE, true, false>), grid, block, lds, st, a);
        return hipGetLastError();
    }
    if (split_waves > 0) return hipErrorInvalidValue;      // the planner splits only 16-byte aligned rows
    dim3 grid(blocks), block(64 * ROWS_WAVES_PER_BLOCK);
    const bool pair = v && nb == 1 && a.p >= 512;
    if constexpr (sizeof(T) == 4) {
        if (!v && nb == 1 && half_vec_ok(4, a.X, a.ldx)) {
            hipLaunchKernelGGL((dense_rows_kernel<T, 1, 2, MODE, false, false>), grid, block, 0, st, a);
            return hipGetLastError();
        }
    }
    if (nb == 1) {
        if (pair) hipLaunchKernelGGL((dense_rows_kernel<T, 1, VEC, MODE, false, true>), grid, block, 0, st, a);
        else if (v) hipLaunchKernelGGL((dense_rows_kernel<T, 1, VEC, MODE, false, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_rows_kernel<T, 1, 1, MODE, false, false>), grid, block, 0, st, a);
    } else {
        if (v) hipLaunchKernelGGL((dense_rows_kernel<T, 2, VEC, MODE, false, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((dense_rows_kernel<T, 2, 1, MODE, false, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

template <typename T> static hipError_t rows_dispatch(const RowsArgs &a, int blocks, int split_waves, hipStream_t st)
{
    switch (a.mode) {
    case ROW_OBJ: return rows_dispatch_mode<T, ROW_OBJ>(a, blocks, split_waves, st);
    case ROW_GRAD: return rows_dispatch_mode<T, ROW_GRAD>(a, blocks, split_waves, st);
    case ROW_PREP: return rows_dispatch_mode<T, ROW_PREP>(a, blocks, split_waves, st);
    case ROW_APPLY: return rows_dispatch_mode<T, ROW_APPLY>(a, blocks, split_waves, st);
    case ROW_PRED: return rows_dispatch_mode<T, ROW_PRED>(a, blocks, split_waves, st);
    case ROW_MARGIN: return a.M2 ? rows_dispatch_mode<T, ROW_MARGIN>(a, blocks, split_waves, st) : hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_dense_rows(int dtype, const RowsArgs &a, int blocks, int split_waves, hipStream_t st)
{
    return dtype == SSN_F32 ? rows_dispatch<float>(a, blocks, split_waves, st) : rows_dispatch<double>(a, blocks, split_waves, st);
}

template <typename T> static hipError_t xtu_dispatch(const XtuArgs &a, hipStream_t st)
{
    constexpr int VEC = 16 / sizeof(T);
    const int nb = (a.K + 15) / 16;
    const bool v = vec_ok<T>(a.X, a.ldx);
    dim3 grid((unsigned)((a.p + 255) / 256), (unsigned)a.nchunks), block(256);
    if (a.Zpart) {
        if (!v || nb != 1 || !a.Pin || !a.zu_part || a.nslices < 1) return hipErrorInvalidValue;
        hipLaunchKernelGGL((dense_xtu_kernel<T, 1, VEC, true>), grid, block, 0, st, a);
        return hipGetLastError();
    }
    if constexpr (sizeof(T) == 4) {
        if (!v && nb == 1 && half_vec_ok(4, a.X, a.ldx)) {
            hipLaunchKernelGGL((dense_xtu_kernel<T, 1, 2>), grid, block, 0, st, a);
            return hipGetLastError();
        }
    }
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

// Fused one-pass kernel: margins, per-row epilogue and (for ROW_GRAD / ROW_APPLY) the transposed
// product, reading every row of X exactly once (eqs. (10)-(13) with both products of Alg. 7 in one
// sweep; same for Alg. 6).
//
// A workgroup owns whole 16-row blocks; its waves split the features into slices of a.fw features
// (a.fw <= min(NLD*LF, NSB*SBF), a multiple of the vector width).  Per row block:
//   1. every lane already holds its part of the wave's 16 x fw tile of X in the A-operand layout
//      (prefetched into registers while the previous block was processed; all loads are unconditional --
//      out-of-slice lanes read a safe address and are zeroed -- so they stay in flight together);
//   2. phase A: Z_partial (16x16) += X_tile * W_slice, W operands from an LDS copy of M;
//   3. the partial margins go to LDS; wave w adds accumulator element v = w (, w + nw, ..) over the waves
//      in a fixed order and does the per-row work for it, so the epilogue runs once per row block;
//   4. U comes back through LDS in accumulator layout, which is the B-operand layout of the transposed
//      product;
//   5. phase C: the wave's X tile is transposed through a wave-private LDS scratch (rows become the
//      contraction index) and G_slice (fw x 16) += X_tile^T * U accumulates in registers.
// At the end each workgroup writes its p x K partial; the finalize kernel adds them in a fixed order.
//
// ONE: every workgroup has at most one row block (sampled products on a few thousand rows).  Each element
// of M is then used once per workgroup, so the lanes load their W operands straight from global memory
// into registers instead of staging M in LDS, and nothing is prefetched for a next block.
template <typename T, int MODE, int NLD, int NSB, int MAXW, bool ONE>
__global__ __launch_bounds__(64 * MAXW) void dense_fused_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef typename V4<T>::type v4;
    constexpr int VEC = 16 / sizeof(T);
    typedef Pack<T, VEC> pack;
    constexpr int LF = 4 * VEC;              // features covered by one vector load of the wave
    constexpr int SBF = 16 * VEC;            // features per transposition sub-block
    constexpr int NT = NSB * VEC;            // 16-feature output tiles of the transposed product
    constexpr int STR = SBF + VEC;           // scratch row stride (elements): 16 bytes of padding
    constexpr bool HAS_C = (MODE == ROW_GRAD || MODE == ROW_APPLY);
    constexpr bool NEED_LAB = (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_PRED);

#ifdef SSN_PROFILE_PHASES
    const long long t_entry = clock64();
    const long long w_entry = wall_clock64();
#endif
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, nw = blockDim.x >> 6;
    const int q = lane & 15, g = lane >> 4;
    const int K = a.K;
    const int64_t p = a.p;
    const int fw = a.fw;
    // LDS copy of M, class-major (wl[c * ws + f], zero beyond p): a lane's operands then sit at constant
    // offsets from one base address.  ws is odd so the class rows start in different banks.
    const int wrows = (nw - 1) * fw + NLD * LF;
    const int ws = wrows | 1;
    T *wl = (T *)smem_raw;
    T *zpart = wl + ((size_t)ws * K + VEC - 1) / VEC * VEC;  // MAXW x 4 x 64 partial margins (16-byte aligned)
    T *zfull = zpart + (size_t)MAXW * 256 * (HAS_C ? 1 : 2); // U of the block (modes with a transposed product)
    T *scr = zfull + 256 + (size_t)w * 16 * STR;             // wave-private transposition scratch
    // The fp64 multi-wave kernels with a transposed product have no register to spare, and the running loss sum
    // and alpha product are touched once per row block by four of the waves: they live in LDS there (a kernel
    // that spills even a few registers uses scratch memory, which costs ~14 us per launch on this machine).
    constexpr bool LDS_ACC = HAS_C && sizeof(T) == 8 && MAXW > 1;
    double *acc_l = (double *)(zfull + 256 + (size_t)(HAS_C ? blockDim.x >> 6 : 0) * 16 * STR) + (w & 3) * 128 + lane;

    const T *X = (const T *)a.X;
    const int fs = w * fw;
    const int64_t fend = (fs + fw < p) ? (int64_t)(fs + fw) : p;   // features [fs, fend) belong to this wave
    const int qc = (q < K) ? q : K - 1;
    const bool cvalid = q < K;
    const T *wlane = wl + qc * ws + fs + VEC * g;            // this lane's B operands: wlane[LF * j + m]
    const int64_t nblk = (a.nrows + 15) / 16;

    // sample position -> data row of the lane's A-operand row of block rb
    auto block_row = [&](int64_t rb) -> int64_t {
        int64_t si = rb * 16 + q;
        if (si >= a.nrows) si = a.nrows - 1;
        return a.S ? (int64_t)a.S[si] : si;
    };
    // tile load: one base address per lane, constant offsets per load; a load is skipped (register keeps its
    // old, finite-or-not contents, which mask_block then replaces) only where it would leave the row's
    // storage of ldx elements, so every issued load is in bounds and none depends on another
    // Rows need no alignment beyond their element's: a vector load of the tile is declared with that alignment
    // (the hardware takes dword-aligned wide loads).  Whole vectors are read, so the last one of a row whose length
    // is not a multiple of the vector width reaches past the row: into the next row on every row but the last of
    // the matrix, which is read from a zero-padded copy the launcher passes (a.tail_row, a.tail_len elements).
    struct __attribute__((packed, aligned(sizeof(T)))) upack { T v[VEC]; };
    // Elements from a lane's first element of a row that may be read: the row's own storage and, where its
    // length is not a multiple of the vector width, the first elements of the next row (32-bit: the comparisons
    // against it cost a register pair and several instructions each in 64 bits, and there is one per load).
    // The last row of the matrix is read from the launcher's copy of it, which is that long.
    const int room = a.tail_len - fs - VEC * g;
    const int last_row = (int)(a.n - 1);                          // row numbers fit 31 bits
    auto row_base = [&](int64_t xr) -> const T * {
        const T *b = ((int)xr == last_row) ? (const T *)a.tail_row : X + xr * a.ldx;
        return b + fs + VEC * g;
    };
    auto load_vec = [&](const T *src, pack &dst) {
        const upack u = *(const upack *)src;
#pragma unroll
        for (int m = 0; m < VEC; ++m) dst.v[m] = u.v[m];
    };
    auto load_block = [&](int64_t xr, pack(&x)[NLD]) {
        const T *xbase = row_base(xr);
#pragma unroll
        for (int j = 0; j < NLD; ++j)
            if (LF * j + VEC <= room) load_vec(xbase + LF * j, x[j]);
    };
    // one vector of the next tile; issued one at a time between the MFMAs of the current block, because a
    // compute unit cannot hold a whole tile of outstanding loads and a wave stalls at issue when it is full
    auto load_one = [&](const T *xbase, int room, int j, pack(&x)[NLD]) {
        if (LF * j + VEC <= room) load_vec(xbase + LF * j, x[j]);
    };
    // this lane's elements LF * j + m of the tile are inside the wave's slice for LF * j + m < nval (one 32-bit
    // register against constants: 64-bit feature indices here cost a register pair per load)
    const int nval = (int)(fend - fs) - VEC * g;
    auto mask_block = [&](pack(&x)[NLD]) {
        const int nv = nval;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
#pragma unroll
            for (int m = 0; m < VEC; ++m) x[j].v[m] = (LF * j + m < nv) ? x[j].v[m] : T(0);
        }
    };

    pack xn[NLD];
    int64_t rb = blockIdx.x;
#pragma unroll
    for (int j = 0; j < NLD; ++j) xn[j] = pack{};
    // A wave's memory counter retires in order, so the prologue issues its loads in the order their results
    // are needed: the row index of the first block, the first batch of M (independent of everything), the
    // first tile (needs the row index), then the small per-row data.
    const int64_t xr0 = (rb < nblk) ? block_row(rb) : 0;

    // LDS copy of M: thread t copies elements t, t + blockDim, .. of the row-major wrows x K block, WB loads in
    // flight at a time; (wf, wc) is the feature / class of the element it copies next
    constexpr int WB = 16;
    const T *M = (const T *)a.M;
    const int wtotal = wrows * K;
    const int wstep_f = (int)blockDim.x / K, wstep_c = (int)blockDim.x - wstep_f * K;
    int wf = tid / K, wc = tid - wf * K, widx = tid;
    // source offset and LDS position of that element, advanced by additions only
    int64_t wsrc = (int64_t)wf * a.ldm + wc;
    int wpos = wc * ws + wf;
    const int64_t wsrc_step = (int64_t)wstep_f * a.ldm + wstep_c, wsrc_wrap = a.ldm - K;
    const int wpos_step = wstep_c * ws + wstep_f, wpos_wrap = 1 - K * ws;
    T wtmp[WB];
    int wdst[WB];
    auto w_load = [&]() {
#pragma unroll
        for (int uu = 0; uu < WB; ++uu) {
            const bool in = widx < wtotal;
            const bool ok = in && wf < p;
            wtmp[uu] = M[ok ? wsrc : 0];
            wdst[uu] = in ? (ok ? wpos : -2 - wpos) : -1;    // >= 0: copy; <= -2: store zero; -1: nothing
            widx += (int)blockDim.x;
            wc += wstep_c;
            wf += wstep_f;
            wsrc += wsrc_step;
            wpos += wpos_step;
            if (wc >= K) {
                wc -= K;
                ++wf;
                wsrc += wsrc_wrap;
                wpos += wpos_wrap;
            }
        }
    };
    auto w_store = [&]() {
#pragma unroll
        for (int uu = 0; uu < WB; ++uu) {
            if (wdst[uu] >= 0) wl[wdst[uu]] = wtmp[uu];
            else if (wdst[uu] <= -2) wl[-2 - wdst[uu]] = T(0);
        }
    };
#ifdef SSN_PROFILE_PHASES
    const long long tp0 = clock64();
#endif
    // ONE: this lane's W operands, M[fs + LF*j + VEC*g + m][qc], zero beyond p
    T bd[ONE ? NLD : 1][VEC];
    if constexpr (ONE) {
        // 32-bit offsets from the uniform base (the launcher admits the one-pass kernel only where p * ldm fits)
        const int f0 = fs + VEC * g, ldm32 = (int)a.ldm, p32 = (int)p;
#pragma unroll
        for (int j = 0; j < NLD; ++j)
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const int ff = f0 + LF * j + m;
                bd[j][m] = M[(unsigned)((ff < p32) ? (ff * ldm32 + qc) : 0)];
            }
    } else {
        w_load();
    }
#ifdef SSN_PROFILE_PHASES
    __builtin_amdgcn_sched_barrier(0);
    const long long tp1 = clock64();
    __builtin_amdgcn_sched_barrier(0);
#endif
    if (rb < nblk) load_block(xr0, xn);
#ifdef SSN_PROFILE_PHASES
    __builtin_amdgcn_sched_barrier(0);
    const long long tp2 = clock64();
    __builtin_amdgcn_sched_barrier(0);
#endif

    // accumulator elements whose per-row work this wave does.  MAXW == 1: the single wave does all four in
    // registers.  Otherwise the workgroup has at least four waves and wave w < 4 does element w.
    constexpr int SLOTS = (MAXW == 1) ? 4 : 1;
    const int nslot = (MAXW == 1) ? 4 : ((w < 4) ? 1 : 0);
    // label / probability of the rows of block rbq this wave's slots cover
    int lab_n[SLOTS];
    T pin_n[SLOTS];
    auto load_meta = [&](int64_t rbq) {
#pragma unroll
        for (int k = 0; k < SLOTS; ++k) {
            lab_n[k] = 0;
            pin_n[k] = T(0);
            if (k < nslot && rbq < nblk) {
                const int v = (MAXW == 1) ? k : w;
                int64_t sv = rbq * 16 + d_row<T>(g, v);
                if (sv >= a.nrows) sv = a.nrows - 1;
                if constexpr (MODE == ROW_APPLY) pin_n[k] = ((const T *)a.Pin)[sv * a.KP + q];
                if constexpr (NEED_LAB) lab_n[k] = a.labels[a.S ? (int64_t)a.S[sv] : sv];
            }
        }
    };
    load_meta(rb);
    // data row of this lane's A-operand row in the NEXT block (needed when that block's loads are issued)
    int64_t xr_n = (rb + gridDim.x < nblk) ? block_row(rb + gridDim.x) : 0;

#ifdef SSN_PROFILE_PHASES
    __builtin_amdgcn_sched_barrier(0);
    const long long tp3 = clock64();
    __builtin_amdgcn_sched_barrier(0);
#endif
    if constexpr (ONE) {
        const int64_t f0 = fs + VEC * g;
#pragma unroll
        for (int j = 0; j < NLD; ++j)
#pragma unroll
            for (int m = 0; m < VEC; ++m) bd[j][m] = (cvalid && f0 + LF * j + m < p) ? bd[j][m] : T(0);
    } else {
        w_store();
        for (int base = WB * (int)blockDim.x; base < wtotal; base += WB * (int)blockDim.x) {
            w_load();
            w_store();
        }
    }
#ifdef SSN_PROFILE_PHASES
    __builtin_amdgcn_sched_barrier(0);
    const long long tp4 = clock64();
    __builtin_amdgcn_sched_barrier(0);
#endif
    if constexpr (!ONE) __syncthreads();

    v4 G[HAS_C ? NT : 1];
#pragma unroll
    for (int t = 0; t < (HAS_C ? NT : 1); ++t) G[t] = v4{0, 0, 0, 0};
    double loss = 0.0, lprod = 1.0;         // sum of the row terms without log(alpha); product of the alphas
    if constexpr (LDS_ACC) {
        if (w < 4) {
            acc_l[0] = 0.0;
            acc_l[64] = 1.0;
        }
    }
    int hits = 0;
    int it = 0;

#ifdef SSN_PROFILE_PHASES
    long long tph[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define SSN_TICK(i) do { __builtin_amdgcn_sched_barrier(0); const long long t_ = clock64(); tph[i] += t_ - tlast; tlast = t_; __builtin_amdgcn_sched_barrier(0); } while (0)
    long long tlast = clock64();
    const long long t_loop = tlast;
#else
#define SSN_TICK(i) do { } while (0)
#endif
    for (; rb < nblk; rb += gridDim.x) {
#ifdef SSN_PROFILE_PHASES
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): time spent waiting for the prefetched tile
        SSN_TICK(0);
#endif
        pack xc[NLD];
#pragma unroll
        for (int j = 0; j < NLD; ++j) xc[j] = xn[j];
        mask_block(xc);
        // The memory counter of a wave retires in order, so a small load issued after bulk prefetch loads
        // would wait for all of them.  Everything small is therefore fetched one block ahead and BEFORE the
        // prefetch of that block is issued: labels / probabilities of block rb+G and the row index of block
        // rb+2G now, the tile of block rb+G (row index already in xr_n) spread over the MFMAs below.
        const int64_t rbn = rb + gridDim.x;
        const bool has_next = rbn < nblk;
        const int64_t xr_next = xr_n;
        int lab_pre[SLOTS];
        T pin_pre[SLOTS];
#pragma unroll
        for (int k = 0; k < SLOTS; ++k) {
            lab_pre[k] = lab_n[k];
            pin_pre[k] = pin_n[k];
        }
        if constexpr (!ONE) {
            load_meta(rbn);
            xr_n = (rbn + gridDim.x < nblk) ? block_row(rbn + gridDim.x) : 0;
        }
        const T *xbase_n = row_base(xr_next);
        const int room_n = has_next ? room : 0;                 // no next block: every load is skipped
        // issued during phase A, the rest in phase C (all of them in phase A, or a quarter, is 2-8 % slower)
        constexpr int LOADS_A = HAS_C ? (NLD + 1) / 2 : NLD;
        constexpr int LOADS_C = (NLD - LOADS_A + NSB - 1) / NSB;          // per transposition sub-block
        SSN_TICK(1);

        // phase A (fp32: two accumulators break the dependent MFMA chain; fp64 has no registers to spare)
        constexpr bool TWO_ACC = sizeof(T) == 4;
        v4 z0 = v4{0, 0, 0, 0}, z1 = v4{0, 0, 0, 0};
        // W operands come from LDS ahead of the MFMAs that use them, through a ring of register sets: two steps
        // ahead where registers allow, one step (a step is VEC MFMAs, longer than an LDS read) in the fp64
        // kernels with a transposed product, which have none to spare
        constexpr int AHEAD = (HAS_C && sizeof(T) == 8) ? 1 : 2;
        constexpr int RING = AHEAD + 1;
        T bq[RING][VEC];
        if constexpr (!ONE) {
#pragma unroll
            for (int jj = 0; jj < AHEAD && jj < NLD; ++jj)
#pragma unroll
                for (int m = 0; m < VEC; ++m) bq[jj][m] = wlane[LF * jj + m];
        }
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            if constexpr (!ONE) {
                if (j + AHEAD < NLD) {
#pragma unroll
                    for (int m = 0; m < VEC; ++m) bq[(j + AHEAD) % RING][m] = wlane[LF * (j + AHEAD) + m];
                }
            }
#pragma unroll
            for (int m = 0; m < VEC; ++m) {
                const T b = ONE ? bd[j][m] : (cvalid ? bq[j % RING][m] : T(0));
                if (TWO_ACC && ((j * VEC + m) & 1)) z1 = mfma16(xc[j].v[m], b, z1);
                else z0 = mfma16(xc[j].v[m], b, z0);
            }
            if constexpr (!ONE) {
                if (j < LOADS_A) load_one(xbase_n, room_n, j, xn);
                __builtin_amdgcn_sched_barrier(0);   // keep this interleaving (and the W reads from piling up)
            }
        }
        v4 z = TWO_ACC ? (z0 + z1) : z0, u = v4{0, 0, 0, 0};
        SSN_TICK(2);
        // sub-block h of the tile goes through the wave's scratch for the transposed product: rows in, columns
        // out.  The first sub-block is written here, before the per-row work, so that its registers are free
        // during it (the fp64 gradient has none to spare).
        auto scr_write = [&](int h) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (4 * h + jj < NLD) *(pack *)(scr + q * STR + LF * jj + VEC * g) = xc[4 * h + jj];
                else *(pack *)(scr + q * STR + LF * jj + VEC * g) = pack{};
        };
        if constexpr (HAS_C) scr_write(0);
        if constexpr (MAXW == 1) {
            bool paired = false;
            if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD) {
                if (K <= 7) {                            // two accumulator elements per pass
                    paired = true;
#pragma unroll
                    for (int v = 0; v < 4; v += 2) {
                        T ub;
                        u[v] = slot_epilogue_pair<T, MODE>(z[v], z[v + 1], ub, a, rb * 16 + d_row<T>(g, v),
                                                           rb * 16 + d_row<T>(g, v + 1), q, lab_pre[v], lab_pre[v + 1], loss, lprod);
                        u[v + 1] = ub;
                    }
                }
            }
            if (!paired) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    u[v] = slot_epilogue<T, MODE>(z[v], a, rb * 16 + d_row<T>(g, v), q, lab_pre[v], pin_pre[v], loss, lprod, hits);
            }
        } else {
            T *zp = zpart + (HAS_C ? 0 : (size_t)(it & 1) * MAXW * 256);
#pragma unroll
            for (int v = 0; v < 4; ++v) zp[(w * 4 + v) * 64 + lane] = z[v];
            __syncthreads();
            SSN_TICK(3);
            {
                if (nslot) {
                    constexpr int k = 0;
                    const int v = w;
                    T sacc = 0;
#pragma unroll
                    for (int ww = 0; ww < MAXW; ++ww) {       // fixed order; waves beyond nw contribute zero
                        const T val = zp[v * 64 + lane + ww * 256];      // slots of absent waves hold stale data
                        sacc += (ww < nw) ? val : T(0);
                    }
                    T uv;
                    if constexpr (LDS_ACC) {
                        double l = acc_l[0], lp = acc_l[64];
                        uv = slot_epilogue<T, MODE, true>(sacc, a, rb * 16 + d_row<T>(g, v), q, lab_pre[k], pin_pre[k], l, lp, hits);
                        acc_l[0] = l;
                        acc_l[64] = lp;
                    } else {
                        uv = slot_epilogue<T, MODE>(sacc, a, rb * 16 + d_row<T>(g, v), q, lab_pre[k], pin_pre[k], loss, lprod,
                                                    hits);
                    }
                    if constexpr (HAS_C) zfull[v * 64 + lane] = uv;
                }
            }
            SSN_TICK(4);
            if constexpr (HAS_C) {
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 4; ++v) u[v] = zfull[v * 64 + lane];
            }
            SSN_TICK(5);
        }
        ++it;

        if constexpr (HAS_C) {
            // sub-block h of the tile goes through the wave's scratch: rows in, columns out.  LDS serves a wave's
            // requests in order, so sub-block h+1 is written as soon as the reads of h are issued and its trip
            // overlaps the MFMAs of h.
#pragma unroll
            for (int h = 0; h < NSB; ++h) {
                __builtin_amdgcn_wave_barrier();
                pack c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) c[i] = *(const pack *)(scr + d_row<T>(g, i) * STR + VEC * q);
                __builtin_amdgcn_wave_barrier();
                if (h + 1 < NSB) scr_write(h + 1);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int m = 0; m < VEC; ++m) G[h * VEC + m] = mfma16(c[i].v[m], u[i], G[h * VEC + m]);
                if constexpr (!ONE) {
#pragma unroll
                    for (int l = 0; l < LOADS_C; ++l)
                        if (LOADS_A + h * LOADS_C + l < NLD) load_one(xbase_n, room_n, LOADS_A + h * LOADS_C + l, xn);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        SSN_TICK(6);
    }
#ifdef SSN_PROFILE_PHASES
    const long long t_loop_end = clock64();
#endif

    if constexpr (HAS_C) {
        // feature of accumulator element v of tile (h, m): fs + h*SBF + VEC*d_row(g, v) + m; the lane part of it
        // goes into one base pointer, the rest is a uniform offset
        // (computed from an opaque copy of the lane's group so that nothing of it is prepared before the loop and
        // carried through it: the fp64 kernels have no register for that, and would spill it to scratch memory)
        int g_out = g, fs_out = fs;
        asm volatile("" : "+v"(g_out), "+v"(fs_out));
        const int lane_row = d_row<T>(g_out, 0);             // d_row(g, v) = lane_row + d_row(0, v)
        T *pl = (T *)a.part + (int64_t)blockIdx.x * p * K + ((int64_t)fs_out + VEC * lane_row) * K + q;
        const int nout = (int)(fend - fs_out) - VEC * lane_row;      // this lane's rows fo of the slice are inside it for fo < nout
#pragma unroll
        for (int h = 0; h < NSB; ++h) {
#pragma unroll
            for (int m = 0; m < VEC; ++m)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int fo = h * SBF + VEC * d_row<T>(0, v) + m;       // uniform
                    if (fo < nout && q < K) pl[(int64_t)fo * K] = G[h * VEC + m][v];
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // four partials per workgroup: wave w < 4 owns the rows of accumulator element w
    if (w < 4) {
        if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
            if constexpr (LDS_ACC) {
                loss = acc_l[0];
                lprod = acc_l[64];
            }
            if constexpr (MODE != ROW_APPLY) loss += log(lprod);
            for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
            if (lane == 0) a.loss_part[blockIdx.x * 4 + w] = loss;
            if (w == 0 && lane > 0 && lane < 4 && lane >= nw) a.loss_part[blockIdx.x * 4 + lane] = 0.0;
        } else if constexpr (MODE == ROW_PRED) {
            for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
            if (lane == 0) a.hit_part[blockIdx.x * 4 + w] = hits;
            if (w == 0 && lane > 0 && lane < 4 && lane >= nw) a.hit_part[blockIdx.x * 4 + lane] = 0;
        }
    }
#ifdef SSN_PROFILE_PHASES
    __builtin_amdgcn_s_waitcnt(0x0F70);
    const long long t_end = clock64();
    const long long w_end = wall_clock64();
    if (blockIdx.x == 3 && lane == 0 && (w == 0 || w == 5)) {
        printf("[phases] mode %d wave %d blocks %d: wait %lld issue %lld A %lld bar1 %lld epi %lld bar2 %lld C %lld cycles\n", MODE,
               w, it, tph[0], tph[1], tph[2], tph[3], tph[4], tph[5], tph[6]);
        printf("[clock] mode %d wave %d: %lld cycles in %lld ns\n", MODE, w, t_end - t_entry, (w_end - w_entry) * 10);
        printf("[timeline] mode %d wave %d: prologue %lld (to M loads %lld, issue M %lld, issue tile %lld, meta %lld, M to LDS %lld, sync %lld) loop %lld store %lld cycles\n",
               MODE, w, t_loop - t_entry, tp0 - t_entry, tp1 - tp0, tp2 - tp1, tp3 - tp2, tp4 - tp3, t_loop - tp4,
               t_loop_end - t_loop, t_end - t_loop_end);
    }
#endif
}

// Register footprints the one-pass kernel is compiled for.  NLD vector loads and NSB transposition
// sub-blocks bound the features a wave can own; MAXW waves per workgroup fix the register budget
// (512 / ceil(MAXW/4) per lane).  Shapes are tried in this order.
struct FusedShape { int nld, nsb, maxw, flags; };
constexpr int SHAPE_NO_C_MULTI = 1;       // multi-wave use only without a transposed product (it would spill)
constexpr int SHAPE_SINGLE_WAVE = 2;      // single-wave workgroups only (a footprint for narrow matrices)
template <typename T> struct FusedTable;
template <> struct FusedTable<double> {
    static constexpr int N = 4;
    // 56 / 72 / 104 / 128 features per wave; ordered by footprint, the first shape that fits serves
    static constexpr FusedShape shape[N] = {{7, 2, 8, SHAPE_SINGLE_WAVE}, {9, 3, 12, SHAPE_NO_C_MULTI}, {13, 4, 8, 0}, {16, 4, 8, 0}};
};
template <> struct FusedTable<float> {
    static constexpr int N = 3;
    static constexpr FusedShape shape[N] = {{4, 1, 8, 0}, {7, 2, 8, 0}, {8, 2, 8, 0}};        // 64 / 112 / 128 features per wave
};
constexpr FusedShape FusedTable<double>::shape[];
constexpr FusedShape FusedTable<float>::shape[];

// Split p features over nw waves of fw features each (fw a multiple of the vector width) and pick the
// instantiation; returns its index in FusedTable<T>, or -1 when no shape fits.
template <typename T> static int fused_shape(int64_t p, bool has_c, int *nw, int *fw)
{
    constexpr int VEC = 16 / sizeof(T);
    constexpr int LF = 4 * VEC, SBF = 16 * VEC;
    for (int i = 0; i < FusedTable<T>::N; ++i) {
        const FusedShape sh = FusedTable<T>::shape[i];
        const int cap = (sh.nld * LF < sh.nsb * SBF) ? sh.nld * LF : sh.nsb * SBF;
        int64_t n = (p + cap - 1) / cap;
        if (n > 1) n = (n + 3) / 4 * 4;              // same number of waves on each of the 4 SIMDs
        if (n > sh.maxw) continue;
        if (n > 1 && (sh.flags & SHAPE_SINGLE_WAVE)) continue;
        if (n > 1 && has_c && (sh.flags & SHAPE_NO_C_MULTI)) continue;
        int f = (int)((p + n - 1) / n);
        f = (f + VEC - 1) / VEC * VEC;
        if (f > cap) continue;
        *nw = (int)n;
        *fw = f;
        return i;
    }
    return -1;
}

template <typename T> static size_t fused_lds_bytes(int nw, int fw, int nld, int maxw, int K, bool has_c)
{
    constexpr int VEC = 16 / sizeof(T);
    constexpr int LF = 4 * VEC, STR = 16 * VEC + VEC;
    const size_t ws = ((size_t)(nw - 1) * fw + (size_t)nld * LF) | 1;
    size_t elems = (ws * K + VEC - 1) / VEC * VEC + (size_t)maxw * 256 * (has_c ? 1 : 2) + 256;
    if (has_c) elems += (size_t)nw * 16 * STR;
    size_t bytes = elems * sizeof(T);
    if (has_c && sizeof(T) == 8 && maxw > 1) bytes += 4 * 128 * sizeof(double);      // loss sums / alpha products of four waves
    return bytes;
}

template <typename T> static bool fused_ok(const RowsArgs &a)
{
    constexpr int VEC = 16 / sizeof(T);
    if (a.K > 16 || (uintptr_t)a.X % sizeof(T) != 0) return false;
    if ((a.p + 256) * a.ldm >= ((int64_t)1 << 31)) return false;         // 32-bit offsets into the p x K operand
    // whole-vector loads: the last vector of a row may reach VEC - 1 elements into the next row, which must exist
    // (the last row's copy, RowsArgs::tail_row, covers the end of the matrix)
    if (a.ldx < VEC) return false;
    for (int c = 0; c < 2; ++c) {            // both kernel families (with / without transposed product) must fit
        int nw, fw;
        const int i = fused_shape<T>(a.p, c == 1, &nw, &fw);
        if (i < 0) return false;
        if (fused_lds_bytes<T>(nw, fw, FusedTable<T>::shape[i].nld, nw == 1 ? 1 : FusedTable<T>::shape[i].maxw, a.K, c == 1) > 160 * 1024)
            return false;
    }
    return true;
}

// Can the one-pass kernel serve this shape?  (one 16-column class tile, rows of at least one vector, a feature
// split that fits one of the compiled register footprints, LDS within the 160 KB of a gfx950 compute unit)
bool dense_fused_supported(int dtype, const RowsArgs &a)
{
    return dtype == SSN_F32 ? fused_ok<float>(a) : fused_ok<double>(a);
}

// dynamic LDS of the launch fused_launch_mode would make (0: no shape fits)
template <typename T> static size_t fused_grid_lds(int64_t p, int K, bool has_c)
{
    int nw, fw;
    const int i = fused_shape<T>(p, has_c, &nw, &fw);
    if (i < 0) return 0;
    return fused_lds_bytes<T>(nw, fw, FusedTable<T>::shape[i].nld, nw == 1 ? 1 : FusedTable<T>::shape[i].maxw, K, has_c);
}

// waves per workgroup the one-pass kernel would use for a.mode
int dense_fused_waves(int dtype, const RowsArgs &a)
{
    if (dense_narrow_applies(dtype, a)) return 1;
    int nw = 1, fw = 0;
    const bool has_c = (a.mode == ROW_GRAD || a.mode == ROW_APPLY);
    if (dtype == SSN_F32) fused_shape<float>(a.p, has_c, &nw, &fw);
    else fused_shape<double>(a.p, has_c, &nw, &fw);
    return nw;
}

int dense_fused_grid(int dtype, const RowsArgs &a, int num_cus)
{
    if (dense_narrow_applies(dtype, a)) return dense_narrow_grid(dtype, a, num_cus);
    int nw = 1, fw = 0;
    const bool has_c = (a.mode == ROW_GRAD || a.mode == ROW_APPLY);
    if (dtype == SSN_F32) fused_shape<float>(a.p, has_c, &nw, &fw);
    else fused_shape<double>(a.p, has_c, &nw, &fw);
    int per_cu = 8 / nw;                          // aim at 8 or more waves per compute unit
    if (per_cu < 1) per_cu = 1;
    // single-wave workgroups without a transposed product fit three to a SIMD (at most 150 registers), and a
    // streaming pass over a narrow matrix wants them all
    if (nw == 1 && !has_c) per_cu = 12;
    // with a transposed product: three fp32 waves to a SIMD still help (581012 x 54 gradient 53 -> 49 us); in fp64 two
    // are the best (75 us against 80 with three)
    if (nw == 1 && has_c && dtype == SSN_F32) per_cu = 12;
    // never more workgroups than stay resident together: the rest would start when the first ones end, as a
    // second, thinly occupied round
    const size_t lds = (dtype == SSN_F32) ? fused_grid_lds<float>(a.p, a.K, has_c) : fused_grid_lds<double>(a.p, a.K, has_c);
    if (lds > 0 && (size_t)per_cu * lds > 160 * 1024) per_cu = (int)(160 * 1024 / lds);
    if (per_cu < 1) per_cu = 1;
    const int64_t nblk = (a.nrows + 15) / 16;
    int64_t grid = (int64_t)num_cus * per_cu;
    if (grid > nblk) grid = nblk;
    if (grid < 1) grid = 1;
    return (int)grid;
}

template <typename T, int MODE, int NLD, int NSB, int MAXW, bool ONE>
static hipError_t fused_launch_kern(const RowsArgs &a, int grid, int nw, size_t lds, hipStream_t st)
{
    auto kern = dense_fused_kernel<T, MODE, NLD, NSB, MAXW, ONE>;
    static size_t lds_allowed = 48 * 1024;          // raise the dynamic LDS limit once per instantiation
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_allowed = 160 * 1024;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * nw), lds, st, a);
    return hipGetLastError();
}

template <typename T, int MODE, int NLD, int NSB, int MAXW>
static hipError_t fused_launch_inst(const RowsArgs &a, int grid, int nw, size_t lds, hipStream_t st)
{
    // the one-block-per-workgroup variant exists for the modes that run on a Hessian sample
    if constexpr (MODE == ROW_APPLY || MODE == ROW_PREP) {
        if ((a.nrows + 15) / 16 <= grid) return fused_launch_kern<T, MODE, NLD, NSB, MAXW, true>(a, grid, nw, lds, st);
    }
    return fused_launch_kern<T, MODE, NLD, NSB, MAXW, false>(a, grid, nw, lds, st);
}

template <typename T, int MODE> static hipError_t fused_launch_mode(RowsArgs a, int grid, hipStream_t st)
{
    typedef FusedTable<T> TB;
    int nw, fw;
    constexpr bool has_c = (MODE == ROW_GRAD || MODE == ROW_APPLY);
    const int i = fused_shape<T>(a.p, has_c, &nw, &fw);
    if (i < 0) return hipErrorInvalidValue;
    a.fw = fw;
    // single-wave workgroups run the MAXW = 1 instantiation: sized for the table's MAXW, its LDS would let only
    // 6 of the 8 workgroups a compute unit is given be resident, and the grid would run in two rounds
    const size_t lds = fused_grid_lds<T>(a.p, a.K, has_c);
#define SSN_FUSED_SHAPE(I, W) fused_launch_inst<T, MODE, TB::shape[I].nld, TB::shape[I].nsb, W>(a, grid, nw, lds, st)
    if (nw == 1) {      // single-wave workgroups: no cross-wave reduction compiled in
        if (i == 0) return SSN_FUSED_SHAPE(0, 1);
        if (i == 1) return SSN_FUSED_SHAPE(1, 1);
        if (i == 2) return SSN_FUSED_SHAPE(2, 1);
        if constexpr (TB::N > 3) return SSN_FUSED_SHAPE(TB::N - 1, 1);
        return hipErrorInvalidValue;
    }
    // multi-wave workgroups: only the (shape, mode) pairs fused_shape can pick are compiled
#define SSN_FUSED_MULTI(I)                                                                                              \
    if constexpr (!(TB::shape[I].flags & SHAPE_SINGLE_WAVE) && !(has_c && (TB::shape[I].flags & SHAPE_NO_C_MULTI))) {  \
        if (i == I) return SSN_FUSED_SHAPE(I, TB::shape[I].maxw);                                                       \
    }
    SSN_FUSED_MULTI(0)
    SSN_FUSED_MULTI(1)
    SSN_FUSED_MULTI(2)
    if constexpr (TB::N > 3) {
        SSN_FUSED_MULTI(TB::N - 1)
    }
#undef SSN_FUSED_MULTI
    return hipErrorInvalidValue;
#undef SSN_FUSED_SHAPE
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
// ROW_OBJ / ROW_GRAD 4 * `grid` loss partials (ROW_APPLY: of sum_i z_i . u_i there), ROW_PRED 4 * `grid` hit partials.
hipError_t launch_dense_fused(int dtype, const RowsArgs &a, int grid, hipStream_t st)
{
    // long passes over narrow matrices: the vector-unit kernel (dense_narrow.hip)
    if (dense_narrow_applies(dtype, a)) return launch_dense_narrow(dtype, a, grid, st);
    if (!a.tail_row || a.tail_len < a.p) return hipErrorInvalidValue;       // the kernel reads row n-1 from this copy
    return dtype == SSN_F32 ? fused_dispatch<float>(a, grid, st) : fused_dispatch<double>(a, grid, st);
}

}  // namespace ssn
