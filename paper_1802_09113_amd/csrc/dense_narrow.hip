// One-pass kernel for long passes over NARROW dense matrices (an even number of at most 64 features, at most
// ten weight columns: the shapes of Table 1's Covertype and Drive Diagnostics sets), entirely on the vector units.
//
// With 54 features a 16 x 16 x 4 matrix-core tile is mostly padding (6 of 16 class columns, 54 of 56 / 64
// features) and, more to the point, the per-row work of eqs. (8), (9), (14)-(17) on margins that sit in the
// accumulator layout (a row spread over 16 lanes) costs more than both products.  Here a wave owns 64 rows at a
// time and every quantity of a row lives in ONE lane:
//   load    : the 64 x p block comes in with one 2-element vector per lane, half a wave per row (32 loads, each
//             covering two whole rows, i.e. contiguous memory), into registers;
//   margins : the block goes through the wave's own LDS tile in two halves of the features and lane r walks row r
//             of the tile; z_rc += x_rf W_fc.  The W operands are the same for every lane, so they are scalar
//             operands: scalar loads through the constant cache (W is a few KB here and stays there), two buffers,
//             the request for step j + 1 placed by hand right behind the wait for step j's -- no vector-memory, LDS
//             or lane traffic for W;
//   row work: eqs. (8), (9), (11), (12), (14)-(17) for 64 rows at once, one row per lane, no cross-lane traffic;
//   X^T U   : the rows of U go to LDS; the transposed product runs from the REGISTERS the block was loaded into:
//             lane (h, l) holds features 2l, 2l+1 of rows 2j + h, G_fc += x_rf u_rc with u_rc a half-wave
//             broadcast from LDS; register j is free once its rows have been used, and the next block's load j goes
//             out right there.  The accumulators stay in registers over all the wave's blocks and leave as one
//             p x K partial per workgroup (added by the finalize kernels in a fixed order: no atomics).
// A workgroup is one wave: nothing here needs a barrier.  Eq. (5), (6) / Alg. 5, 6 and eqs. (10)-(13) / Alg. 7, 8
// as in the matrix-core kernels; results differ from theirs by the order of summation only.
#include "ssn_internal.h"
#include "ssn_math.h"

#include <limits>
#include <stdlib.h>
#include <string.h>

namespace ssn {

namespace {

__device__ __forceinline__ float n_exp(float x) { return expf(x); }
// (an opaque zero keeps the routine's sixteen 64-bit coefficients from being set up once and held in registers across
// the kernel, whose fp64 forms have none to spare)
__device__ __forceinline__ double n_exp(double x) { return exp_nonpos(x, opaque_zero()); }

__device__ __forceinline__ double n_rcp(double a)          // a in [1, 17]: estimate plus two Newton steps
{
    double x = __builtin_amdgcn_rcp(a);
    x = fma(fma(-a, x, 1.0), x, x);
    x = fma(fma(-a, x, 1.0), x, x);
    return x;
}
__device__ __forceinline__ float n_rcp(float a)
{
    float x = __builtin_amdgcn_rcpf(a);
    x = fmaf(fmaf(-a, x, 1.0f), x, x);
    return x;
}

template <typename T> struct alignas(2 * sizeof(T)) NPair { T v[2]; };

constexpr int NARROW_ROWS = 64;          // rows per block: one per lane
constexpr int NARROW_MAX_P = 64;         // 32 lanes x 2 elements per row
constexpr int NARROW_MAX_K = 10;
#define SSN_CONSTANT __attribute__((address_space(4)))

// The tile goes through LDS in two halves of the features (pairs [0, ph) and [ph, p2), ph = ceil(p2 / 2) <= HP): a
// whole 64 x p block of fp64 would leave room for one wave per SIMD only, and this kernel needs a second one to fill
// the gaps of the first.  Row stride 2 HP elements with HP odd: with a lane per row, the lanes of a wide LDS access
// hit every bank once.
template <typename T, int K, int MODE, int HP>
__global__ __launch_bounds__(64) void dense_narrow_kernel(RowsArgs a)
{
    if (a.skip && *a.skip) return;
    typedef NPair<T> pair;
    struct __attribute__((packed, aligned(sizeof(T)))) upair { T v[2]; };      // rows are element-aligned only
    constexpr bool HAS_C = (MODE == ROW_GRAD || MODE == ROW_APPLY);
    constexpr bool NEED_LAB = (MODE == ROW_OBJ || MODE == ROW_GRAD);
    constexpr int KU = K + (K & 1);          // row stride of the U tile: whole pairs
    constexpr int NLD = NARROW_ROWS / 2;     // loads per lane and block
    constexpr int HS = 2 * HP;               // row stride of the tile (elements)

    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *xs = (T *)smem_raw;                   // 64 rows of half the features
    T *us = xs + NARROW_ROWS * HS;           // 64 rows of U, stride KU

    const int lane = threadIdx.x, h = lane >> 5, lp = lane & 31;
    const int p2 = (int)(a.p >> 1), ph = (p2 + 1) >> 1;
    const bool act = lp < p2;                // this lane holds a pair of features
    const char *Xb = (const char *)a.X;
    const uint32_t ldxb = (uint32_t)(a.ldx * (int64_t)sizeof(T));        // the launcher checks that it fits
    const int nrows = (int)a.nrows;          // row counts fit 31 bits
    const int nblk = (nrows + NARROW_ROWS - 1) / NARROW_ROWS;
    const T SSN_CONSTANT *Wc = (const T SSN_CONSTANT *)a.M;
    const int ldm = (int)a.ldm;

    pair xn[NLD];
    // lanes beyond the last pair of features repeat its load (in bounds, same cache line) so that no load is
    // conditional; what they load is never used
    const uint32_t voff = (uint32_t)(act ? lp : p2 - 1) * (uint32_t)(2 * sizeof(T));
    // load j of a block brings rows 2j (lower half of the wave) and 2j + 1 (upper half); their numbers come from the
    // lanes that own them in the per-row phases (rowl: this lane's data row of that block)
    auto load_one = [&](int rowl, int j) {
        const int r0 = __builtin_amdgcn_readlane(rowl, 2 * j), r1 = __builtin_amdgcn_readlane(rowl, 2 * j + 1);
        const uint32_t r = (uint32_t)(h ? r1 : r0);
        const upair u = *(const upair *)(Xb + ((uint64_t)r * ldxb + voff));
        xn[j].v[0] = u.v[0];
        xn[j].v[1] = u.v[1];
    };
    // sample position -> data row, clamped so that every load stays inside the matrix
    auto block_row = [&](int rb) -> int {
        int si = rb * NARROW_ROWS + lane;
        si = si < nrows ? si : nrows - 1;
        return a.S ? a.S[si] : si;
    };

    T G[2][K];
#pragma unroll
    for (int c = 0; c < K; ++c) G[0][c] = G[1][c] = T(0);
    double loss = 0.0, lprod = 1.0;

    // margins of the tile's pairs [j0, j1) (tile-local index j - j0).  The W operands are the same for every lane:
    // scalar loads (constant cache) into scalar registers, no vector-memory or LDS traffic.  Scalar loads return out
    // of order, so a wait for one is a wait for all: the operands of pair j + 1 (two rows of W, and the lane's two
    // elements from LDS) are requested right after the wait for pair j's and arrive while pair j is multiplied.
    T z[K];
    auto margins = [&](int j0, int j1) {
        const T *xrow = xs + lane * HS;
        T w[2][2 * K];
        pair xv[2];
        auto request = [&](int j, int b) {
            const int jc = j < j1 ? j : j1 - 1;              // past the end: the last pair again (never multiplied)
            const T SSN_CONSTANT *wr = Wc + (int64_t)(2 * jc) * ldm;
#pragma unroll
            for (int c = 0; c < K; ++c) w[b][c] = wr[c];
#pragma unroll
            for (int c = 0; c < K; ++c) w[b][K + c] = wr[ldm + c];
            xv[b] = *(const pair *)(xrow + 2 * (jc - j0));
        };
        auto multiply = [&](int b) {
#pragma unroll
            for (int c = 0; c < K; ++c) z[c] = fma(xv[b].v[0], w[b][c], z[c]);
#pragma unroll
            for (int c = 0; c < K; ++c) z[c] = fma(xv[b].v[1], w[b][K + c], z[c]);
        };
        request(j0, 0);
        int j = j0;
        for (; j + 1 < j1; j += 2) {
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): pair j is here
            __builtin_amdgcn_sched_barrier(0);
            request(j + 1, 1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(0);
            __builtin_amdgcn_s_waitcnt(0xC07F);              // pair j + 1 is here
            __builtin_amdgcn_sched_barrier(0);
            request(j + 2, 0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(1);
        }
        if (j < j1) {                                        // an odd pair is left, requested last
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_sched_barrier(0);
            multiply(0);
        }
    };

    int rb = blockIdx.x;
    int rowc = 0, labc = 0;                  // this lane's data row and label in the current block
    if (rb < nblk) {
        rowc = block_row(rb);
        if constexpr (NEED_LAB) labc = a.labels[rowc];
#pragma unroll
        for (int j = 0; j < NLD; ++j) load_one(rowc, j);
    }
    while (rb < nblk) {
        const int sv = rb * NARROW_ROWS + lane;              // sample position of this lane's row
        const bool valid = sv < nrows;
        // the block after this one (the wave's last block stands in for itself where a row number is needed)
        const int rbn = rb + (int)gridDim.x;
        const bool more = rbn < nblk;
        const int rown = block_row(more ? rbn : rb);
        int labn = 0;
        if constexpr (NEED_LAB) labn = a.labels[rown];

#pragma unroll
        for (int c = 0; c < K; ++c) z[c] = T(0);
        // first half of the features -> LDS (the previous reads of the tile were issued before: LDS serves a wave
        // in order), margins; then the second half
        __builtin_amdgcn_wave_barrier();
        if (lp < ph) {
#pragma unroll
            for (int j = 0; j < NLD; ++j) *(pair *)(xs + (2 * j + h) * HS + 2 * lp) = xn[j];
        }
        __builtin_amdgcn_wave_barrier();
        margins(0, ph);
        __builtin_amdgcn_wave_barrier();
        if (lp >= ph && act) {
#pragma unroll
            for (int j = 0; j < NLD; ++j) *(pair *)(xs + (2 * j + h) * HS + 2 * (lp - ph)) = xn[j];
        }
        __builtin_amdgcn_wave_barrier();
        if constexpr (!HAS_C) {
            // nothing reads the registers of this block again: the next block's loads go out now
            if (more) {
#pragma unroll
                for (int j = 0; j < NLD; ++j) load_one(rown, j);
            }
        }
        if (p2 > ph) margins(ph, p2);

        // per-row work
        T u[K];
        if constexpr (MODE == ROW_APPLY) {
            // (the probabilities are fetched here, not ahead of the margins: with nine and ten weight columns in fp64
            // the registers they would hold through the margins are what keeps a second wave off the SIMD)
            T pin[K];
            const T *pr = (const T *)a.Pin + (int64_t)(valid ? sv : 0) * a.KP;
#pragma unroll
            for (int c = 0; c < K; ++c) pin[c] = pr[c];
            T t = T(0);
#pragma unroll
            for (int c = 0; c < K; ++c) t = fma(pin[c], z[c], t);
            T zu = T(0);
#pragma unroll
            for (int c = 0; c < K; ++c) {
                u[c] = valid ? (pin[c] * z[c] - pin[c] * t) : T(0);          // eq. (12)
                zu = fma(z[c], u[c], zu);
            }
            loss += (double)zu;                              // sum_i z_i . u_i: the curvature term of Alg. 2
        } else {
            // eqs. (8), (9): M = max{0, z_c}, alpha = e^{-M} + sum_c e^{z_c - M}
            T Mx = T(0);
#pragma unroll
            for (int c = 0; c < K; ++c) Mx = fmax(Mx, z[c]);
            T alpha = n_exp(-Mx);
            T e[K];
#pragma unroll
            for (int c = 0; c < K; ++c) {
                e[c] = n_exp(z[c] - Mx);
                alpha += e[c];
            }
            const T inv = n_rcp(alpha);
            if constexpr (MODE == ROW_PREP) {
                if (valid) {
                    T *pw = (T *)a.UP + (int64_t)sv * a.KP;
                    for (int c = K; c < a.KP; ++c) pw[c] = T(0);
#pragma unroll
                    for (int c = 0; c < K; ++c) pw[c] = e[c] * inv;           // eq. (11)
                }
            } else {
                // eqs. (14)-(17): the row adds M + log(alpha) - z_label; the logarithm is taken of a running
                // product of the alphas (each in [1, C]), folded into the sum before it can overflow
                T lin = T(0);
#pragma unroll
                for (int c = 0; c < K; ++c) lin = (labc == c) ? z[c] : lin;
                if (valid) {
                    loss += (double)Mx - (double)lin;
                    lprod *= (double)alpha;
                }
                if (lprod > 1e250) {
                    loss += log_ge1(lprod, opaque_zero());
                    lprod = 1.0;
                }
                if constexpr (MODE == ROW_GRAD) {
#pragma unroll
                    for (int c = 0; c < K; ++c) u[c] = valid ? (e[c] * inv - ((labc == c) ? T(1) : T(0))) : T(0);
                }
            }
        }

        if constexpr (HAS_C) {
            // U -> LDS, then the transposed product from the registers the block was loaded into: lane (h, lp) holds
            // features 2 lp, 2 lp + 1 of rows 2 j + h; u_rc is broadcast from LDS.  Register j is free once its row
            // has been used: the next block's load j goes out right there.
            T *urow = us + lane * KU;
#pragma unroll
            for (int c = 0; c < K; ++c) urow[c] = u[c];
            if constexpr (KU > K) urow[K] = T(0);
            __builtin_amdgcn_wave_barrier();
            // (the wave's last block has no next one: the same loop without the loads)
            auto xtu_step = [&](int j) {
                const T *ur = us + (2 * j + h) * KU;
                const T x0 = xn[j].v[0], x1 = xn[j].v[1];     // lanes without features: sums nobody reads
#pragma unroll
                for (int c2 = 0; c2 < KU / 2; ++c2) {
                    const pair uu = *(const pair *)(ur + 2 * c2);
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int c = 2 * c2 + i;
                        if (c < K) {
                            G[0][c] = fma(x0, uu.v[i], G[0][c]);
                            G[1][c] = fma(x1, uu.v[i], G[1][c]);
                        }
                    }
                }
            };
            if (more) {
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    xtu_step(j);
                    load_one(rown, j);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NLD; ++j) xtu_step(j);
            }
        }
        if (!more) break;
        rb = rbn;
        rowc = rown;
        labc = labn;
    }

    if constexpr (HAS_C) {
        // the two halves of the wave hold the even and the odd rows' sums of the same features
#pragma unroll
        for (int c = 0; c < K; ++c) {
            G[0][c] += __shfl_xor(G[0][c], 32);
            G[1][c] += __shfl_xor(G[1][c], 32);
        }
        if (h == 0 && act) {
            T *pl = (T *)a.part + (int64_t)blockIdx.x * a.p * K + (int64_t)(2 * lp) * K;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                pl[c] = G[0][c];
                pl[K + c] = G[1][c];
            }
        }
    }
    if constexpr (MODE == ROW_OBJ || MODE == ROW_GRAD || MODE == ROW_APPLY) {
        if constexpr (MODE != ROW_APPLY) loss += log_ge1(lprod, opaque_zero());
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
        // four partials per workgroup, as the multi-wave kernels leave them
        if (lane < 4) a.loss_part[blockIdx.x * 4 + lane] = (lane == 0) ? loss : 0.0;
    }
}

// pair slots per row of the tile (odd, at least the pairs of a half): 15 serves p <= 60, 17 the rest
int narrow_half_pairs(int64_t p) { return p <= 60 ? 15 : 17; }

template <typename T> size_t narrow_lds_bytes(int64_t p, int K, bool has_c)
{
    const int ku = K + (K & 1);
    return ((size_t)NARROW_ROWS * 2 * narrow_half_pairs(p) + (has_c ? (size_t)NARROW_ROWS * ku : 0)) * sizeof(T);
}

typedef void (*narrow_fn)(RowsArgs);

template <typename T, int K, int HP> narrow_fn narrow_kernel_kh(int mode)
{
    switch (mode) {
    case ROW_OBJ: return dense_narrow_kernel<T, K, ROW_OBJ, HP>;
    case ROW_GRAD: return dense_narrow_kernel<T, K, ROW_GRAD, HP>;
    case ROW_PREP: return dense_narrow_kernel<T, K, ROW_PREP, HP>;
    case ROW_APPLY: return dense_narrow_kernel<T, K, ROW_APPLY, HP>;
    default: return nullptr;
    }
}

template <typename T, int K> narrow_fn narrow_kernel_k(int mode, int hp)
{
    return hp == 15 ? narrow_kernel_kh<T, K, 15>(mode) : narrow_kernel_kh<T, K, 17>(mode);
}

template <typename T> narrow_fn narrow_kernel_t(int K, int mode, int hp)
{
    switch (K) {
    case 1: return narrow_kernel_k<T, 1>(mode, hp);
    case 2: return narrow_kernel_k<T, 2>(mode, hp);
    case 3: return narrow_kernel_k<T, 3>(mode, hp);
    case 4: return narrow_kernel_k<T, 4>(mode, hp);
    case 5: return narrow_kernel_k<T, 5>(mode, hp);
    case 6: return narrow_kernel_k<T, 6>(mode, hp);
    case 7: return narrow_kernel_k<T, 7>(mode, hp);
    case 8: return narrow_kernel_k<T, 8>(mode, hp);
    case 9: return narrow_kernel_k<T, 9>(mode, hp);
    case 10: return narrow_kernel_k<T, 10>(mode, hp);
    default: return nullptr;
    }
}

narrow_fn narrow_kernel(int dtype, const RowsArgs &a)
{
    const int hp = narrow_half_pairs(a.p);
    return dtype == SSN_F32 ? narrow_kernel_t<float>(a.K, a.mode, hp) : narrow_kernel_t<double>(a.K, a.mode, hp);
}

size_t narrow_lds(int dtype, const RowsArgs &a)
{
    const bool has_c = (a.mode == ROW_GRAD || a.mode == ROW_APPLY);
    return dtype == SSN_F32 ? narrow_lds_bytes<float>(a.p, a.K, has_c) : narrow_lds_bytes<double>(a.p, a.K, has_c);
}

// workgroups of a launch that stay resident on one compute unit together (registers and LDS), asked of the runtime
// once per kernel and LDS size
int narrow_resident_per_cu(int dtype, const RowsArgs &a)
{
    static int cache[2][NARROW_MAX_K + 1][8][2];             // [dtype][K][mode][tile width], 0 = not asked yet
    const int hp = narrow_half_pairs(a.p);
    int &slot = cache[dtype == SSN_F32 ? 0 : 1][a.K][a.mode & 7][hp == 15 ? 0 : 1];
    if (slot == 0) {
        int n = 0;
        const narrow_fn k = narrow_kernel(dtype, a);
        if (!k || hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void *)k, 64, narrow_lds(dtype, a)) != hipSuccess || n < 1) n = 4;
        slot = n;
    }
    return slot;
}

// 0: by the size of the pass (default), 1: whenever the shape allows it, -1: never (SSN_NARROW_PATH=on / off)
int narrow_forced()
{
    const char *e = getenv("SSN_NARROW_PATH");         // read at every call: tests switch it
    if (!e) return 0;
    if (strcmp(e, "on") == 0) return 1;
    if (strcmp(e, "off") == 0) return -1;
    return 0;
}

}  // namespace

// Does the vector-unit kernel serve this launch?  Shape: an even number of at most 64 features, at most ten weight
// columns.  Mode: the two with a transposed product; the margins-only passes are as fast (objective) or faster (the
// probabilities of eq. (11), whose rows this kernel writes lane by lane) through the matrix-core kernel and take this
// one only where SSN_NARROW_PATH=on asks for it.  Size, measured on 54 / 48 / 30 features (gradient and product over n
// rows, microseconds, this kernel / the matrix-core one): from NARROW_MIN_ROWS rows on -- on a few thousand sampled rows
// a wave's single 64-row block is one long chain (product on 5810 rows 11.0 / 9.0, on 20000 rows 11.9 / 14.3, on 50000
// rows 19.4 / 21.6 in fp64); and in fp64 with many weight columns, where the accumulators and the block leave the
// product one wave per SIMD (K >= 9) or little room (K = 8), only up to NARROW_BIG_K_ROWS rows: product with K = 8
// 19.5 / 22.1 on 50000 rows but 59.7 / 57.4 on 400000, K = 10 22.6 / 22.5 and 73.0 / 57.3; gradient with K = 9 65.1 /
// 68.8 on 400000 rows, K = 10 20.1 / 24.7 on 50000 and 70.9 / 69.6 on 400000.  fp32 wins at every K (K = 10: 46.1 /
// 51.7 on 400000 rows).
constexpr int64_t NARROW_MIN_ROWS = 16384, NARROW_BIG_K_ROWS = 100000;
bool dense_narrow_applies(int dtype, const RowsArgs &a)
{
    const int forced = narrow_forced();
    if (forced < 0) return false;
    if (a.p < 2 || a.p > NARROW_MAX_P || (a.p & 1) || a.K < 1 || a.K > NARROW_MAX_K) return false;
    if (a.mode != ROW_OBJ && a.mode != ROW_GRAD && a.mode != ROW_PREP && a.mode != ROW_APPLY) return false;
    if (a.nrows < 1 || a.nrows >= ((int64_t)1 << 31) - 2 * NARROW_ROWS || a.n >= ((int64_t)1 << 31)) return false;
    const size_t es = dtype == SSN_F32 ? 4 : 8;
    if ((uintptr_t)a.X % es != 0 || (uintptr_t)a.M % es != 0 || a.ldx * (int64_t)es >= ((int64_t)1 << 30)) return false;
    if (forced > 0) return true;
    if ((a.mode != ROW_GRAD && a.mode != ROW_APPLY) || a.nrows < NARROW_MIN_ROWS) return false;
    if (dtype != SSN_F32 && a.nrows > NARROW_BIG_K_ROWS && a.K >= (a.mode == ROW_APPLY ? 8 : 10)) return false;
    return true;
}

// workgroups (single waves): as many as stay resident together (LDS bound, at most ten per compute unit), in
// whole rounds -- every wave gets the same number of blocks, give or take one
int dense_narrow_grid(int dtype, const RowsArgs &a, int num_cus)
{
    int per_cu = narrow_resident_per_cu(dtype, a);
    if (per_cu > 12) per_cu = 12;
    const int64_t nblk = (a.nrows + NARROW_ROWS - 1) / NARROW_ROWS;
    const int64_t resident = (int64_t)num_cus * per_cu;
    if (nblk <= resident) return (int)(nblk < 1 ? 1 : nblk);
    const int64_t rounds = (nblk + resident - 1) / resident;
    return (int)((nblk + rounds - 1) / rounds);
}

int dense_narrow_max_grid(int64_t p, int num_cus) { return (p >= 2 && p <= NARROW_MAX_P && !(p & 1)) ? num_cus * 12 : 0; }

hipError_t launch_dense_narrow(int dtype, const RowsArgs &a, int grid, hipStream_t st)
{
    const narrow_fn k = narrow_kernel(dtype, a);
    if (!k) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k, dim3(grid), dim3(64), narrow_lds(dtype, a), st, a);
    return hipGetLastError();
}

}  // namespace ssn
