// fp64 exponential and logarithm on the ranges the stable log-sum-exp needs (device code, shared by the dense
// and the CSR kernels).
#pragma once
#include <hip/hip_runtime.h>

namespace ssn {

// The stable log-sum-exp of eq. (8), (9) only ever exponentiates non-positive numbers and only takes the
// logarithm of alpha in [1, C].  On those ranges short fp64 routines (argument reduction + Taylor /
// atanh series, errors of a few 1e-16) need far fewer registers than the general library calls, which
// matters inside the MFMA kernels.
// `zero` is 0.0 that the compiler cannot see through (see opaque_zero): added to every coefficient it keeps the
// sixteen 64-bit constants from being set up once before the caller's loop and held in registers across it.
// The fp64 gradient kernel has no register for that; it would spill one, and a kernel that touches scratch
// memory at all pays ~14 us per launch on this machine.  Adding 0.0 changes no value.
__device__ __forceinline__ double exp_nonpos(double x, double zero)
{
    if (x < -745.2) return 0.0;                                   // underflow, and -inf
    const double n = rint(x * (1.4426950408889634 + zero));
    double r = fma(n, -6.93147180369123816490e-01 + zero, x);     // x - n*ln2, ln2 split in two parts
    r = fma(n, -1.90821492927058770002e-10 + zero, r);
    double t = 1.0 / 6227020800.0 + zero;                         // sum_{k<=13} r^k / k!, |r| <= ln2/2
    t = fma(t, r, 1.0 / 479001600.0 + zero);
    t = fma(t, r, 1.0 / 39916800.0 + zero);
    t = fma(t, r, 1.0 / 3628800.0 + zero);
    t = fma(t, r, 1.0 / 362880.0 + zero);
    t = fma(t, r, 1.0 / 40320.0 + zero);
    t = fma(t, r, 1.0 / 5040.0 + zero);
    t = fma(t, r, 1.0 / 720.0 + zero);
    t = fma(t, r, 1.0 / 120.0 + zero);
    t = fma(t, r, 1.0 / 24.0 + zero);
    t = fma(t, r, 1.0 / 6.0 + zero);
    t = fma(t, r, 0.5);
    t = fma(t, r, 1.0);
    t = fma(t, r, 1.0);
    return ldexp(t, (int)n);
}
__device__ __forceinline__ double opaque_zero()
{
    double z = 0.0;
    asm volatile("" : "+v"(z));
    return z;
}
// log a for a >= 1; `zero` as in exp_nonpos
__device__ __forceinline__ double log_ge1(double a, double zero)
{
    int k;
    double m = frexp(a, &k);                                      // a = m * 2^k, m in [0.5, 1)
    if (m < 0.70710678118654752) { m *= 2.0; k -= 1; }            // m in [sqrt(1/2), sqrt(2))
    const double s = (m - 1.0) / (m + 1.0), s2 = s * s;           // log m = 2 atanh(s), |s| <= 0.1716
    double t = 1.0 / 23.0 + zero;
    t = fma(t, s2, 1.0 / 21.0 + zero);
    t = fma(t, s2, 1.0 / 19.0 + zero);
    t = fma(t, s2, 1.0 / 17.0 + zero);
    t = fma(t, s2, 1.0 / 15.0 + zero);
    t = fma(t, s2, 1.0 / 13.0 + zero);
    t = fma(t, s2, 1.0 / 11.0 + zero);
    t = fma(t, s2, 1.0 / 9.0 + zero);
    t = fma(t, s2, 1.0 / 7.0 + zero);
    t = fma(t, s2, 1.0 / 5.0 + zero);
    t = fma(t, s2, 1.0 / 3.0 + zero);
    t = fma(t, s2, 1.0);
    return fma((double)k, 0.69314718055994530942 + zero, 2.0 * s * t);
}
__device__ __forceinline__ double log_ge1(double a) { return log_ge1(a, 0.0); }

// x shifted along the wave by a DPP control word, lanes without a source lane (and rows or banks masked out) get 0
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_or_zero(double x)
{
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}
// inclusive sum over the lanes of a wave: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of rows 0 and
// 2 is added to the rows behind them (row_bcast:15 into rows 1 and 3) and lane 31 to the upper half (row_bcast:31)
__device__ __forceinline__ double wave_inclusive_scan(double x)
{
    x += dpp_or_zero<0x111, 0xf>(x);
    x += dpp_or_zero<0x112, 0xf>(x);
    x += dpp_or_zero<0x114, 0xf>(x);
    x += dpp_or_zero<0x118, 0xf>(x);
    x += dpp_or_zero<0x142, 0xa>(x);
    x += dpp_or_zero<0x143, 0xc>(x);
    return x;
}

}  // namespace ssn
