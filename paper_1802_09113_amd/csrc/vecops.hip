// Level-1 style kernels on p x K blocks (the paper's d-vectors), the fixed-order reducers, the
// validation passes and the device-resident conjugate-gradient steps of Alg. 2.
//
// All reductions are two-stage and deterministic: every block writes one partial, consumers add the
// partials in one fixed order.  Scalars of Alg. 2 never visit the host: each kernel of product k reads
// the state slot k and block 0 writes slot k+1, so no slot is read and written by the same launch.
#include "ssn_internal.h"
#include "ssn_math.h"

namespace ssn {

// sum over the block's VEC_BLOCK threads, the same bits in every thread: a butterfly inside each wave,
// then the four wave sums in order
__device__ __forceinline__ double block_sum(double v)
{
    __shared__ double sm[VEC_BLOCK / 64];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = sm[0];
#pragma unroll
    for (int k = 1; k < VEC_BLOCK / 64; ++k) r += sm[k];
    __syncthreads();
    return r;
}

// two sums at once (same order of operations as block_sum for each)
__device__ __forceinline__ void block_sum2(double a, double b, double &ra, double &rb)
{
    __shared__ double sm2[2 * (VEC_BLOCK / 64)];
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        b += __shfl_xor(b, off);
    }
    if ((threadIdx.x & 63) == 0) {
        sm2[threadIdx.x >> 6] = a;
        sm2[VEC_BLOCK / 64 + (threadIdx.x >> 6)] = b;
    }
    __syncthreads();
    ra = sm2[0];
    rb = sm2[VEC_BLOCK / 64];
#pragma unroll
    for (int k = 1; k < VEC_BLOCK / 64; ++k) {
        ra += sm2[k];
        rb += sm2[VEC_BLOCK / 64 + k];
    }
    __syncthreads();
}

// this thread's share of part[0..n): elements threadIdx.x, + VEC_BLOCK, .. added in that order, eight loads in
// flight at a time (a narrow matrix leaves ten thousand partials, and one load per trip is a chain of round trips)
__device__ __forceinline__ double thread_parts(const double *part, int n)
{
    double v = 0.0;
    for (int i0 = threadIdx.x; i0 < n; i0 += 8 * VEC_BLOCK) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * VEC_BLOCK;
            t[u] = part[i < n ? i : i0];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i0 + u * VEC_BLOCK < n) v += t[u];
    }
    return v;
}

__device__ __forceinline__ double sum_parts(const double *part, int n) { return block_sum(thread_parts(part, n)); }

// offset of element e of a p x K block with leading dimension ld
__device__ __forceinline__ int64_t off_of(int64_t e, int K, int64_t ld)
{
    if (ld == K) return e;
    const int64_t j = e / K;
    return j * ld + (e - j * K);
}

int vec_blocks(int64_t total)
{
    // small blocks: one element per thread (the kernels on them are chains of a few dependent round trips,
    // not bandwidth); large ones: four per thread and a grid-stride loop beyond RED_MAX_PARTS blocks
    const int per_thread = total <= (int64_t)VEC_BLOCK * 256 ? 1 : 4;
    int64_t b = (total + VEC_BLOCK * per_thread - 1) / (VEC_BLOCK * per_thread);
    if (b > RED_MAX_PARTS) b = RED_MAX_PARTS;
    if (b < 1) b = 1;
    return (int)b;
}

// sum over chunks cl, cl + CLN, .. of element e of the per-chunk partials, eight loads in flight at a time,
// added in chunk order
// (skip, s0: the first `skip` of them are already added up in s0)
template <typename T, int CLN>
__device__ __forceinline__ double chunk_sum(const T *part, int nchunks, int64_t total, int64_t e, int cl, int skip = 0,
                                            double s0 = 0.0)
{
    double s = s0;
    for (int c = cl + skip * CLN; c < nchunks; c += 8 * CLN) {
        T v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int cc = c + u * CLN;
            v[u] = part[(int64_t)(cc < nchunks ? cc : cl) * total + e];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (c + u * CLN < nchunks) ? (double)v[u] : 0.0;
    }
    return s;
}

// ---- finalize: out = scale * sum_chunks part + lambda * M -----------------------------------
// A block owns EL consecutive elements at a time; its 256/EL thread rows split the chunk sum and are
// folded through LDS in a fixed order.
template <typename T, int EL> __global__ __launch_bounds__(VEC_BLOCK) void finalize_kernel(FinArgs a)
{
    if (a.skip && *a.skip) return;
    constexpr int CLN = VEC_BLOCK / EL;
    __shared__ double sm[VEC_BLOCK];
    const int el = threadIdx.x % EL, cl = threadIdx.x / EL;
    const int64_t total = a.p * a.K;
    const int64_t ngroups = (total + EL - 1) / EL;
    const T *part = (const T *)a.part;
    const T *M = (const T *)a.M;
    T *out = (T *)a.out;
    double local = 0.0;
    for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int64_t e = grp * EL + el;
        double s = 0.0;
        if (e < total) s = chunk_sum<T, CLN>(part, a.nchunks, total, e, cl);
        sm[threadIdx.x] = s;
        __syncthreads();
        if (cl == 0 && e < total) {
            double t = 0.0;
#pragma unroll
            for (int k = 0; k < CLN; ++k) t += sm[k * EL + el];
            const double m = (double)M[off_of(e, a.K, a.ldm)];
            const T o = (T)(a.scale * t + a.lambda * m);
            out[off_of(e, a.K, a.ldo)] = o;
            local += (double)o * m;
        }
        __syncthreads();
    }
    if (a.dot_part) {
        const double r = block_sum(local);
        if (threadIdx.x == 0) a.dot_part[blockIdx.x] = r;
    }
}

// elements per block: wide rows of partials are read in long contiguous runs, small ones use more
// chunk lanes per element
static int finalize_el(int64_t total) { return total >= 32768 ? 32 : (total >= 2048 ? 16 : 4); }

int finalize_blocks(int64_t p, int K)
{
    const int64_t total = p * K;
    const int el = finalize_el(total);
    int64_t b = (total + el - 1) / el;
    if (b > RED_MAX_PARTS) b = RED_MAX_PARTS;
    return (int)b;
}

template <typename T> static void finalize_launch(const FinArgs &a, int blocks, hipStream_t st)
{
    const int el = finalize_el(a.p * a.K);
    if (el == 32) hipLaunchKernelGGL((finalize_kernel<T, 32>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a);
    else if (el == 16) hipLaunchKernelGGL((finalize_kernel<T, 16>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a);
    else hipLaunchKernelGGL((finalize_kernel<T, 4>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a);
}

hipError_t launch_finalize(int dtype, const FinArgs &a, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32) finalize_launch<float>(a, blocks, st);
    else finalize_launch<double>(a, blocks, st);
    return hipGetLastError();
}

// State before product k from the state before product k-1 and r_k.r_k: lines 10-11 of Alg. 2 for the
// residual product k-1 left (best-iterate test, theta test).  Every thread of every block computes the same.
__device__ __forceinline__ CgSlot cg_advance(const CgSlot &prev, double rr_new, double theta)
{
    const bool ended = prev.done || prev.brk;
    const bool broke = prev.brk && !prev.done;
    const double rnorm = sqrt(rr_new);
    const bool better = !ended && rnorm <= prev.rbest;
    const bool stop = !ended && rnorm <= theta * prev.gnorm;
    CgSlot n;                                       // every field by selects (no branch, no copy of the struct)
    n.rr = ended ? prev.rr : rr_new;
    n.rbest = better ? rnorm : prev.rbest;
    n.gnorm = prev.gnorm;
    n.done = (ended || stop) ? 1 : 0;
    n.iters = (ended && !broke) ? prev.iters : prev.iters + 1;
    n.flags = prev.flags | (stop ? 1 : 0) | (broke ? 2 : 0);
    n.brk = 0;
    n.alpha = 0.0;
    n.best_cur = 0;
    n.best_pending = better ? 1 : 0;
    n.sHs = prev.sHs;
    n.goff = 0.0;
    n.rho = n.sigma = n.pi = n.pibest = 0.0;
    return n;
}

// three sums at once (same order of operations as block_sum for each)
__device__ __forceinline__ void block_sum3(double a, double b, double c, double &ra, double &rb, double &rc)
{
    __shared__ double sm3[3 * (VEC_BLOCK / 64)];
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        b += __shfl_xor(b, off);
        c += __shfl_xor(c, off);
    }
    constexpr int NWV = VEC_BLOCK / 64;
    if ((threadIdx.x & 63) == 0) {
        sm3[threadIdx.x >> 6] = a;
        sm3[NWV + (threadIdx.x >> 6)] = b;
        sm3[2 * NWV + (threadIdx.x >> 6)] = c;
    }
    __syncthreads();
    ra = sm3[0];
    rb = sm3[NWV];
    rc = sm3[2 * NWV];
#pragma unroll
    for (int k = 1; k < NWV; ++k) {
        ra += sm3[k];
        rb += sm3[NWV + k];
        rc += sm3[2 * NWV + k];
    }
    __syncthreads();
}

// Dense paths: the sum of the product's partials and lines 7-12 of Alg. 2 in one launch, two launches per
// CG iteration (product, this).  Two things make that possible.
//
// The product is applied to the residual, not to the search direction.  H is linear, so with
// s_k = r_k + beta s_{k-1} (line 12)  H s_k = H r_k + beta H s_{k-1}: the product's launch needs r_k only,
// which the previous finalize has already written, and never waits for beta; H s_k is kept as a vector
// and updated here, next to s_k itself.
//
// No dot product waits for a vector either.  With Z = X_S r and U the rows of eq. (12),
// r^T (X_S^T U) = sum_i z_i . u_i, which the product's own launch leaves as per-wave partials; the previous
// finalize left the partials of r_k.r_k and r_k.(H s_{k-1}).  So every block knows, before it touches its
// elements: beta = r_k.r_k / r_{k-1}.r_{k-1}, r_k^T H r_k = scale * sum z.u + lambda r_k.r_k,
// s_k^T H s_k = r^T H r + 2 beta r_k.(H s_{k-1}) + beta^2 s_{k-1}^T H s_{k-1}, alpha, and the outcome of the
// tests of lines 10-11 for r_k.  It then sums its elements of X_S^T U and updates H s, s, p_best, p, r for
// them in one go.  Block 0 records the state for the host and for the launches that follow.
//
// The theta test for r_k is only known here, after product k has been launched: when the loop stops, that
// one product has run for nothing (the launches after it see the flag and return at once).
template <typename T, int EL> __global__ __launch_bounds__(VEC_BLOCK) void finalize_cg_kernel(FinArgs a, FinCgArgs g)
{
    // Loads first: the state, this thread's share of the partial sums and the first batch of the block's chunk
    // partials are all independent, so they go out together and the kernel waits once.
    constexpr int CLN = VEC_BLOCK / EL;
    const int el = threadIdx.x % EL, cl = threadIdx.x / EL;
    const int64_t total = a.p * a.K;
    const T *part = (const T *)a.part;
    const CgSlot prev = g.first ? *g.cur : *g.prev;    // k == 0 with n_gg > 0: not the state yet, every use is overridden
    const double *rin = g.first ? g.gg_part : g.rr_in;
    const int nin = g.first ? g.n_gg : g.n_in;
    double vz = 0.0, vr = 0.0, vh = 0.0, tfirst = 0.0;   // tfirst: chunks cl, cl + CLN, .. (first eight) of the first group
    {
        double z4[4], r2[2], h2[2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = threadIdx.x + u * VEC_BLOCK;
            z4[u] = g.zu_part[i < g.n_zu ? i : 0];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = threadIdx.x + u * VEC_BLOCK;
            const bool in = i < nin;
            r2[u] = in ? rin[i] : 0.0;
            h2[u] = (in && !g.first) ? g.rhs_in[i] : 0.0;
        }
        T first[8];
        const int64_t ef = (int64_t)blockIdx.x * EL + el;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int cc = cl + u * CLN;
            first[u] = part[(int64_t)(cc < a.nchunks ? cc : 0) * total + (ef < total ? ef : 0)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) vz += (threadIdx.x + u * VEC_BLOCK < (unsigned)g.n_zu) ? z4[u] : 0.0;
        for (int i = threadIdx.x + 4 * VEC_BLOCK; i < g.n_zu; i += VEC_BLOCK) vz += g.zu_part[i];
        vr = r2[0] + r2[1];
        vh = h2[0] + h2[1];
        for (int i = threadIdx.x + 2 * VEC_BLOCK; i < nin; i += VEC_BLOCK) {
            vr += rin[i];
            if (!g.first) vh += g.rhs_in[i];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) tfirst += (cl + u * CLN < a.nchunks) ? (double)first[u] : 0.0;
    }
    double zu, rr_sum, rhs;
    block_sum3(vz, vr, vh, zu, rr_sum, rhs);
    CgSlot c = cg_advance(prev, rr_sum, g.theta);
    if (g.first) {                                    // the state before product 0: line 1 of Alg. 2 (r_0 = -g)
        const bool fresh = g.n_gg > 0;                // from the partials of g.g, else the initialisation's as it is
        const double gn = sqrt(rr_sum);
        c.rr = fresh ? rr_sum : prev.rr;
        c.rbest = fresh ? gn : prev.rbest;
        c.gnorm = fresh ? gn : prev.gnorm;
        c.done = fresh ? (rr_sum == 0.0 ? 1 : 0) : prev.done;
        c.iters = fresh ? 0 : prev.iters;
        c.flags = fresh ? 0 : prev.flags;
        c.best_pending = 0;
    }
    const double beta = (g.first || c.done) ? 0.0 : c.rr / prev.rr;
    const double rHr = a.scale * zu + a.lambda * c.rr;
    const double sHs = g.first ? rHr : rHr + 2.0 * beta * rhs + beta * beta * prev.sHs;
    const bool brk = !c.done && !(sHs > 0.0);        // not positive definite in floating point: stop, keep p_best
    const double alpha = (c.done || brk) ? 0.0 : c.rr / sHs;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        CgSlot *w = g.cur;                            // field by field: a struct temporary would live in scratch memory
        w->rr = c.rr;
        w->rbest = c.rbest;
        w->gnorm = c.gnorm;
        w->done = c.done;
        w->iters = c.iters;
        w->flags = c.flags;
        w->brk = brk ? 1 : 0;
        w->alpha = alpha;
        w->best_cur = 0;
        w->best_pending = c.best_pending;
        w->sHs = sHs;
        w->goff = 0.0;
        w->rho = w->sigma = w->pi = w->pibest = 0.0;
        if (g.trace) {
            if (!g.first && !prev.done && !prev.brk) g.trace[3 * (g.k - 1) + 1] = sqrt(rr_sum);
            if (!c.done) {
                g.trace[3 * g.k] = alpha;
                g.trace[3 * g.k + 2] = sHs;
                if (brk) g.trace[3 * g.k + 1] = sqrt(c.rr);
            }
        }
    }
    if (!c.best_pending && (c.done || brk)) return;
    __shared__ double sm[VEC_BLOCK];
    const int64_t ngroups = (total + EL - 1) / EL;
    T *pv = (T *)g.pv, *r = (T *)g.r, *sv = (T *)g.s, *hsv = (T *)g.hs, *pb = (T *)g.pbest;
    const bool update = !c.done && !brk;
    double lrr = 0.0, lrh = 0.0;
    for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int64_t e = grp * EL + el;
        double t = 0.0;
        if (update && e < total) {
            if (grp == blockIdx.x) t = chunk_sum<T, CLN>(part, a.nchunks, total, e, cl, 8, tfirst);
            else t = chunk_sum<T, CLN>(part, a.nchunks, total, e, cl);
        }
        sm[threadIdx.x] = t;
        __syncthreads();
        if (cl == 0 && e < total) {
            const int64_t o = off_of(e, a.K, a.ldm);
            const T pe = pv[o];
            if (c.best_pending) pb[o] = pe;                           // line 10 for the iterate the last product left
            if (update) {
                double tt = 0.0;
#pragma unroll
                for (int k = 0; k < CLN; ++k) tt += sm[k * EL + el];
                const double re = (double)r[o];
                const T hr = (T)(a.scale * tt + a.lambda * re);       // the element of H r, rounded as if stored
                const T hs = g.first ? hr : (T)((double)hr + beta * (double)hsv[o]);
                const T sn = g.first ? (T)re : (T)(re + beta * (double)sv[o]);      // line 12
                hsv[o] = hs;
                sv[o] = sn;
                pv[o] = (T)((double)pe + alpha * (double)sn);         // line 8
                const T rn = (T)(re - alpha * (double)hs);            // line 9
                r[o] = rn;
                lrr += (double)rn * (double)rn;
                lrh += (double)rn * (double)hs;
            }
        }
        __syncthreads();
    }
    if (!update) return;
    double rr_o, rh_o;
    block_sum2(lrr, lrh, rr_o, rh_o);
    if (threadIdx.x == 0) {
        g.rr_out[blockIdx.x] = rr_o;
        g.rhs_out[blockIdx.x] = rh_o;
    }
}

template <typename T> static void finalize_cg_launch(const FinArgs &a, const FinCgArgs &g, int blocks, hipStream_t st)
{
    const int el = finalize_el(a.p * a.K);
    if (el == 32) hipLaunchKernelGGL((finalize_cg_kernel<T, 32>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a, g);
    else if (el == 16) hipLaunchKernelGGL((finalize_cg_kernel<T, 16>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a, g);
    else hipLaunchKernelGGL((finalize_cg_kernel<T, 4>), dim3(blocks), dim3(VEC_BLOCK), 0, st, a, g);
}

hipError_t launch_finalize_cg(int dtype, const FinArgs &a, const FinCgArgs &g, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32) finalize_cg_launch<float>(a, g, blocks, st);
    else finalize_cg_launch<double>(a, g, blocks, st);
    return hipGetLastError();
}

// After the last product of the dense paths: lines 10-11 for r_T, the pending copy p_best <- p, the final state.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_tail_kernel(CgVecs v, const CgSlot *prev_p, CgSlot *fin, const double *rr_in,
                                                             int n_in, double theta, double *trace, int k)
{
    const CgSlot prev = *prev_p;
    const double rr_sum = sum_parts(rr_in, n_in);
    const CgSlot c = cg_advance(prev, rr_sum, theta);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        fin->rr = c.rr;
        fin->rbest = c.rbest;
        fin->gnorm = c.gnorm;
        fin->done = c.done;
        fin->iters = c.iters;
        fin->flags = c.flags;
        fin->brk = 0;
        fin->alpha = 0.0;
        fin->best_cur = 0;
        fin->best_pending = 0;
        fin->sHs = c.sHs;
        fin->goff = 0.0;
        fin->rho = fin->sigma = fin->pi = fin->pibest = 0.0;
        if (trace && !prev.done && !prev.brk) trace[3 * (k - 1) + 1] = sqrt(rr_sum);
    }
    if (!c.best_pending) return;
    const int64_t total = v.p * v.K;
    const T *pw = (const T *)v.pv;
    T *pb = (T *)v.pbest;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        pb[o] = pw[o];
    }
}

// The tail for ssn_solve: the final state and the pending p_best copy as in cg_tail_kernel, then what the iteration
// does next with the direction -- the slope <p_best, g> and the first trial point W + p_best, all from one pass over
// the vectors.  One block (blocks of a few hundred elements) also publishes F(x_k), the slope and the state to
// host-visible memory; several blocks leave slope partials and solve_publish_kernel follows.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_tail_solve_kernel(CgVecs v, const CgSlot *prev_p, CgSlot *fin,
                                                                   const double *rr_in, int n_in, double theta, double *trace,
                                                                   int k, const T *W, T *trial, const double *f_dev,
                                                                   double *slope_dev, double *host_out, double *slope_part)
{
    const CgSlot prev = *prev_p;
    const double rr_sum = sum_parts(rr_in, n_in);
    const CgSlot c = cg_advance(prev, rr_sum, theta);
    const int64_t total = v.p * v.K;
    const T *pw = (const T *)v.pv, *G = (const T *)v.G;
    T *pb = (T *)v.pbest;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        T d;
        if (c.best_pending) {
            d = pw[o];
            pb[o] = d;
        } else {
            d = pb[o];
        }
        trial[o] = (T)(1.0 * (double)d + (double)W[o]);       // the arithmetic of the axpy kernel at alpha = 1
        local += (double)d * (double)G[o];
    }
    const double slope = block_sum(local);
    if (threadIdx.x == 0 && gridDim.x > 1) slope_part[blockIdx.x] = slope;       // several blocks: solve_publish_kernel follows
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        fin->rr = c.rr;
        fin->rbest = c.rbest;
        fin->gnorm = c.gnorm;
        fin->done = c.done;
        fin->iters = c.iters;
        fin->flags = c.flags;
        fin->brk = 0;
        fin->alpha = 0.0;
        fin->best_cur = 0;
        fin->best_pending = 0;
        fin->sHs = c.sHs;
        fin->goff = 0.0;
        fin->rho = fin->sigma = fin->pi = fin->pibest = 0.0;
        if (trace && !prev.done && !prev.brk) trace[3 * (k - 1) + 1] = sqrt(rr_sum);
        if (gridDim.x > 1) return;
        *slope_dev = slope;
        host_out[0] = *f_dev;
        host_out[1] = slope;
        // the state for the host, field by field (the struct above may not be visible to this thread's loads yet)
        CgSlot *h = (CgSlot *)(host_out + 2);
        h->rr = c.rr;
        h->rbest = c.rbest;
        h->gnorm = c.gnorm;
        h->done = c.done;
        h->iters = c.iters;
        h->flags = c.flags;
        h->brk = 0;
        h->alpha = 0.0;
        h->best_cur = 0;
        h->best_pending = 0;
        h->sHs = c.sHs;
        h->goff = 0.0;
        h->rho = h->sigma = h->pi = h->pibest = 0.0;
    }
}

hipError_t launch_cg_tail_solve(int dtype, const CgVecs &v, const CgSlot *prev, CgSlot *fin, const double *rr_in, int n_in,
                                double theta, double *trace, int k, const void *W, void *trial, const double *f_dev,
                                double *slope_dev, double *host_out, double *slope_part, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_tail_solve_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, prev, fin, rr_in, n_in, theta,
                           trace, k, (const float *)W, (float *)trial, f_dev, slope_dev, host_out, slope_part);
    else
        hipLaunchKernelGGL(cg_tail_solve_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, prev, fin, rr_in, n_in, theta,
                           trace, k, (const double *)W, (double *)trial, f_dev, slope_dev, host_out, slope_part);
    if (blocks > 1) return launch_solve_publish(slope_part, blocks, f_dev, fin, slope_dev, host_out, false, st);
    return hipGetLastError();
}

hipError_t launch_cg_tail(int dtype, const CgVecs &v, const CgSlot *prev, CgSlot *fin, const double *rr_in, int n_in,
                          double theta, double *trace, int k, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_tail_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, prev, fin, rr_in, n_in, theta, trace, k);
    else
        hipLaunchKernelGGL(cg_tail_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, prev, fin, rr_in, n_in, theta, trace,
                           k);
    return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void scale_copy_kernel(int64_t p, int K, double lambda, const T *M, int64_t ldm,
                                                                T *out, int64_t ldo, const int32_t *skip)
{
    if (skip && *skip) return;
    const int64_t total = p * K;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK)
        out[off_of(e, K, ldo)] = (T)(lambda * (double)M[off_of(e, K, ldm)]);
}

hipError_t launch_scale_copy(int dtype, int64_t p, int K, double lambda, const void *M, int64_t ldm, void *out,
                             int64_t ldo, const int32_t *skip, hipStream_t st)
{
    const int blocks = vec_blocks(p * K) * 4 > 4096 ? 4096 : vec_blocks(p * K) * 4;
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(scale_copy_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, lambda, (const float *)M,
                           ldm, (float *)out, ldo, skip);
    else
        hipLaunchKernelGGL(scale_copy_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, lambda,
                           (const double *)M, ldm, (double *)out, ldo, skip);
    return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void dot_part_kernel(int64_t p, int K, const T *A, int64_t lda, const T *B,
                                                              int64_t ldb, double *part, const int32_t *skip)
{
    if (skip && *skip) return;
    const int64_t total = p * K;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK)
        local += (double)A[off_of(e, K, lda)] * (double)B[off_of(e, K, ldb)];
    const double r = block_sum(local);
    if (threadIdx.x == 0) part[blockIdx.x] = r;
}

hipError_t launch_dot_part(int dtype, int64_t p, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
                           double *part, int blocks, const int32_t *skip, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(dot_part_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (const float *)A, lda,
                           (const float *)B, ldb, part, skip);
    else
        hipLaunchKernelGGL(dot_part_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (const double *)A, lda,
                           (const double *)B, ldb, part, skip);
    return hipGetLastError();
}

template <typename T> __global__ __launch_bounds__(VEC_BLOCK) void pad_copy_kernel(const T *src, int64_t n, T *dst, int64_t len)
{
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < len; e += (int64_t)gridDim.x * VEC_BLOCK)
        dst[e] = e < n ? src[e] : T(0);
}

hipError_t launch_pad_copy(int dtype, const void *src, int64_t n, void *dst, int64_t len, hipStream_t st)
{
    const int blocks = (int)((len + VEC_BLOCK - 1) / VEC_BLOCK);
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(pad_copy_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, (const float *)src, n, (float *)dst, len);
    else
        hipLaunchKernelGGL(pad_copy_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, (const double *)src, n, (double *)dst, len);
    return hipGetLastError();
}

// The paper stacks the weight columns, x = [x_1; ...; x_K] (Sec. 3.3): element (j, c) of the p x K block is
// element c * p + j of that d-vector.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void vec_layout_kernel(int64_t p, int K, T *vec, T *block, int64_t ld, int to_block)
{
    const int64_t total = p * K;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t j = e / K;
        const int c = (int)(e - j * K);
        if (to_block) block[j * ld + c] = vec[(int64_t)c * p + j];
        else vec[(int64_t)c * p + j] = block[j * ld + c];
    }
}

hipError_t launch_vec_layout(int dtype, int64_t p, int K, void *vec, void *block, int64_t ld, bool to_block,
                             hipStream_t st)
{
    const int blocks = vec_blocks(p * (int64_t)K);
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(vec_layout_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (float *)vec, (float *)block, ld,
                           to_block ? 1 : 0);
    else
        hipLaunchKernelGGL(vec_layout_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (double *)vec, (double *)block,
                           ld, to_block ? 1 : 0);
    return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void axpy_kernel(int64_t p, int K, double alpha, const T *X, int64_t ldx,
                                                          const T *Z, int64_t ldz, T *Y, int64_t ldy)
{
    const int64_t total = p * K;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK)
        Y[off_of(e, K, ldy)] = (T)(alpha * (double)X[off_of(e, K, ldx)] + (double)Z[off_of(e, K, ldz)]);
}

// the same, leaving one partial of ||Y||^2 per block: the objective at Y needs it and Y is in registers here
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void axpy_sq_kernel(int64_t p, int K, double alpha, const T *X, int64_t ldx,
                                                             const T *Z, int64_t ldz, T *Y, int64_t ldy, double *sq_part)
{
    const int64_t total = p * K;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const T y = (T)(alpha * (double)X[off_of(e, K, ldx)] + (double)Z[off_of(e, K, ldz)]);
        Y[off_of(e, K, ldy)] = y;
        local += (double)y * (double)y;
    }
    const double sum = block_sum(local);
    if (threadIdx.x == 0) sq_part[blockIdx.x] = sum;
}

hipError_t launch_axpy_sq(int dtype, int64_t p, int K, double alpha, const void *X, int64_t ldx_, const void *Z,
                          int64_t ldz, void *Y, int64_t ldy, double *sq_part, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(axpy_sq_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, alpha, (const float *)X, ldx_,
                           (const float *)Z, ldz, (float *)Y, ldy, sq_part);
    else
        hipLaunchKernelGGL(axpy_sq_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, alpha, (const double *)X,
                           ldx_, (const double *)Z, ldz, (double *)Y, ldy, sq_part);
    return hipGetLastError();
}

hipError_t launch_axpy(int dtype, int64_t p, int K, double alpha, const void *X, int64_t ldx_, const void *Z,
                       int64_t ldz, void *Y, int64_t ldy, hipStream_t st)
{
    const int blocks = vec_blocks(p * K) * 4 > 4096 ? 4096 : vec_blocks(p * K) * 4;
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(axpy_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, alpha, (const float *)X, ldx_,
                           (const float *)Z, ldz, (float *)Y, ldy);
    else
        hipLaunchKernelGGL(axpy_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, alpha, (const double *)X,
                           ldx_, (const double *)Z, ldz, (double *)Y, ldy);
    return hipGetLastError();
}

// A scalar result for a host that is waiting for it: the value into host-visible memory, then (ordered behind it
// at system scope) the ticket the host is spinning on.  The host sees the ticket a microsecond or two after the
// store, without the wake-up latency of a stream synchronisation (~20 us on this machine).
__device__ __forceinline__ void post_to_host(double value, double *out_host, unsigned long long *ticket_host,
                                             unsigned long long ticket)
{
    if (!out_host) return;
    *(volatile double *)out_host = value;
    if (ticket_host) {
        __threadfence_system();
        __hip_atomic_store(ticket_host, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

__global__ __launch_bounds__(VEC_BLOCK) void combine_kernel(const double *a, int na, double scale, const double *b,
                                                             int nb, double coef, double *out, double *out_host,
                                                             unsigned long long *ticket_host, unsigned long long ticket)
{
    const double sa = sum_parts(a, na);
    const double sb = (b != nullptr) ? sum_parts(b, nb) : 0.0;
    if (threadIdx.x == 0) {
        const double v = scale * sa + coef * sb;
        *out = v;
        post_to_host(v, out_host, ticket_host, ticket);
    }
}

// f = scale * sum(loss partials) + half_lambda * ||W||^2 in ONE launch for small blocks: the single block adds
// up the squares of W itself (eight elements per thread in flight), and mirrors the value into host-visible
// memory (nullable) so that the caller only has to wait for the stream, not for a copy
// (sixteen waves: the block's one pass over W and over the partials is a chain of trips to memory, eight loads per
// thread and trip, and with four waves a block of 27 648 weights took fourteen trips)
constexpr int OBJ_BLOCK = 1024;
template <typename T>
__global__ __launch_bounds__(OBJ_BLOCK) void objective_value_kernel(const double *loss_part, int nparts, double scale,
                                                                     const T *W, int64_t p, int K, int64_t ldw,
                                                                     double half_lambda, double *out, double *out_host,
                                                                     unsigned long long *ticket_host,
                                                                     unsigned long long ticket)
{
    const int64_t total = p * K;
    double sq = 0.0;
    for (int64_t e0 = threadIdx.x; e0 < total; e0 += 8 * OBJ_BLOCK) {
        T w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t e = e0 + (int64_t)u * OBJ_BLOCK;
            w[u] = W[off_of(e < total ? e : e0, K, ldw)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (e0 + (int64_t)u * OBJ_BLOCK < total) sq += (double)w[u] * (double)w[u];
    }
    double loss = 0.0;
    for (int i0 = threadIdx.x; i0 < nparts; i0 += 8 * OBJ_BLOCK) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * OBJ_BLOCK;
            t[u] = loss_part[i < nparts ? i : i0];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i0 + u * OBJ_BLOCK < nparts) loss += t[u];
    }
    // the block's two sums: over the lanes of a wave, then over the waves in wave order
    __shared__ double sm[2 * (OBJ_BLOCK / 64)];
    for (int off = 32; off > 0; off >>= 1) {
        loss += __shfl_xor(loss, off);
        sq += __shfl_xor(sq, off);
    }
    if ((threadIdx.x & 63) == 0) {
        sm[threadIdx.x >> 6] = loss;
        sm[OBJ_BLOCK / 64 + (threadIdx.x >> 6)] = sq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sl = sm[0], ss = sm[OBJ_BLOCK / 64];
#pragma unroll
        for (int k = 1; k < OBJ_BLOCK / 64; ++k) {
            sl += sm[k];
            ss += sm[OBJ_BLOCK / 64 + k];
        }
        const double f = scale * sl + half_lambda * ss;
        *out = f;
        post_to_host(f, out_host, ticket_host, ticket);
    }
}

hipError_t launch_objective_value(int dtype, const double *loss_part, int nparts, double scale, const void *W, int64_t p,
                                  int K, int64_t ldw, double half_lambda, double *out, double *out_host,
                                  unsigned long long *ticket_host, unsigned long long ticket, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(objective_value_kernel<float>, dim3(1), dim3(OBJ_BLOCK), 0, st, loss_part, nparts, scale,
                           (const float *)W, p, K, ldw, half_lambda, out, out_host, ticket_host, ticket);
    else
        hipLaunchKernelGGL(objective_value_kernel<double>, dim3(1), dim3(OBJ_BLOCK), 0, st, loss_part, nparts, scale,
                           (const double *)W, p, K, ldw, half_lambda, out, out_host, ticket_host, ticket);
    return hipGetLastError();
}

// ---- line search on cached margins -----------------------------------------------------------------------
// F(W + alpha P) needs the margins X (W + alpha P) = X W + alpha X P: with Z = [X W | X P] kept from one pass over
// the data, a trial of Alg. 3 is a pass over n x 2K numbers instead of over X.  A thread takes a row: eqs. (8), (9),
// (14)-(17) in fp64 on z = zw + alpha zp; one loss partial per block.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void ls_trial_kernel(const T *Z, int kp, int64_t n, int K, const int32_t *labels,
                                                              double alpha, double *loss_part)
{
    double local = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < n; i += (int64_t)gridDim.x * VEC_BLOCK) {
        const T *z = Z + i * kp;
        const int lab = labels[i];
        double Mx = 0.0, lin = 0.0;
        for (int c = 0; c < K; ++c) {
            const double zc = (double)z[c] + alpha * (double)z[K + c];
            Mx = fmax(Mx, zc);
            lin = (c == lab) ? zc : lin;
        }
        double al = exp_nonpos(-Mx, 0.0);
        for (int c = 0; c < K; ++c) al += exp_nonpos((double)z[c] + alpha * (double)z[K + c] - Mx, 0.0);
        local += Mx + log_ge1(al) - lin;
    }
    const double r = block_sum(local);
    if (threadIdx.x == 0) loss_part[blockIdx.x] = r;
}

hipError_t launch_ls_trial(int dtype, const void *Z, int kp, int64_t n, int K, const int32_t *labels, double alpha,
                           double *loss_part, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(ls_trial_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, (const float *)Z, kp, n, K, labels, alpha,
                           loss_part);
    else
        hipLaunchKernelGGL(ls_trial_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, (const double *)Z, kp, n, K, labels,
                           alpha, loss_part);
    return hipGetLastError();
}

// partials of A.A, A.B and B.B from one pass over the two blocks: part[b], part[nb + b], part[2 nb + b]
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void dot3_part_kernel(int64_t p, int K, const T *A, int64_t lda, const T *B, int64_t ldb,
                                                               double *part)
{
    const int64_t total = p * K;
    double aa = 0.0, ab = 0.0, bb = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const double x = (double)A[off_of(e, K, lda)], y = (double)B[off_of(e, K, ldb)];
        aa += x * x;
        ab += x * y;
        bb += y * y;
    }
    double raa, rab;
    block_sum2(aa, ab, raa, rab);
    const double rbb = block_sum(bb);
    if (threadIdx.x == 0) {
        part[blockIdx.x] = raa;
        part[gridDim.x + blockIdx.x] = rab;
        part[2 * gridDim.x + blockIdx.x] = rbb;
    }
}

hipError_t launch_dot3_part(int dtype, int64_t p, int K, const void *A, int64_t lda, const void *B, int64_t ldb, double *part,
                            int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(dot3_part_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (const float *)A, lda,
                           (const float *)B, ldb, part);
    else
        hipLaunchKernelGGL(dot3_part_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, p, K, (const double *)A, lda,
                           (const double *)B, ldb, part);
    return hipGetLastError();
}

// ||W + alpha P||^2 = W.W + 2 alpha W.P + alpha^2 P.P from the partials of the three products
__global__ __launch_bounds__(VEC_BLOCK) void ls_value_kernel(const double *loss_part, int nparts, double scale,
                                                              const double *dots, int nd, double alpha, double half_lambda,
                                                              double *out, double *out_host, unsigned long long *ticket_host,
                                                              unsigned long long ticket)
{
    const double sl = sum_parts(loss_part, nparts);
    const double ww = sum_parts(dots, nd), wp = sum_parts(dots + nd, nd), pp = sum_parts(dots + 2 * nd, nd);
    if (threadIdx.x == 0) {
        const double f = scale * sl + half_lambda * (ww + 2.0 * alpha * wp + alpha * alpha * pp);
        *out = f;
        post_to_host(f, out_host, ticket_host, ticket);
    }
}

hipError_t launch_ls_value(const double *loss_part, int nparts, double scale, const double *dots, int nd, double alpha,
                           double half_lambda, double *out, double *out_host, unsigned long long *ticket_host,
                           unsigned long long ticket, hipStream_t st)
{
    hipLaunchKernelGGL(ls_value_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, loss_part, nparts, scale, dots, nd, alpha, half_lambda,
                       out, out_host, ticket_host, ticket);
    return hipGetLastError();
}

// What the host needs after the CG solve of an SSN iteration, in one launch and without a copy: the slope
// <P, G> from its partials (also left in *slope_dev), F(x_k) from *f_dev and the final CG state, written to
// host-visible memory (host_out: two doubles, then the CgSlot).  The caller only waits for the stream.
__global__ __launch_bounds__(VEC_BLOCK) void solve_publish_kernel(const double *slope_part, int n, const double *f_dev,
                                                                   const CgSlot *fin, double *slope_dev, double *host_out,
                                                                   int support_only)
{
    // support_only: the partials cover the sample's columns; elsewhere the direction is pibest * g
    double slope = sum_parts(slope_part, n);
    if (support_only) slope += fin->pibest * fin->goff;
    if (threadIdx.x == 0) {
        *slope_dev = slope;
        host_out[0] = *f_dev;
        host_out[1] = slope;
    }
    constexpr int NWORDS = (int)(sizeof(CgSlot) / sizeof(int32_t));
    if ((int)threadIdx.x < NWORDS) ((int32_t *)(host_out + 2))[threadIdx.x] = ((const int32_t *)fin)[threadIdx.x];
}

hipError_t launch_solve_publish(const double *slope_part, int n, const double *f_dev, const CgSlot *fin, double *slope_dev,
                                double *host_out, bool support_only, hipStream_t st)
{
    hipLaunchKernelGGL(solve_publish_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, slope_part, n, f_dev, fin, slope_dev, host_out,
                       support_only ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_combine(const double *a, int na, double scale, const double *b, int nb, double coef, double *out,
                          hipStream_t st, double *out_host, unsigned long long *ticket_host, unsigned long long ticket)
{
    hipLaunchKernelGGL(combine_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, a, na, scale, b, nb, coef, out, out_host, ticket_host,
                       ticket);
    return hipGetLastError();
}

__global__ __launch_bounds__(VEC_BLOCK) void sum_int_kernel(const int32_t *a, int na, int32_t *out)
{
    __shared__ long long sm[VEC_BLOCK];
    long long v = 0;
    for (int i = threadIdx.x; i < na; i += VEC_BLOCK) v += a[i];
    sm[threadIdx.x] = v;
    __syncthreads();
    for (int s = VEC_BLOCK / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sm[threadIdx.x] += sm[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (int32_t)sm[0];
}

hipError_t launch_sum_int(const int32_t *a, int na, int32_t *out, hipStream_t st)
{
    hipLaunchKernelGGL(sum_int_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, a, na, out);
    return hipGetLastError();
}

// ---- plain streaming read of a buffer: the practical HBM ceiling next to which the kernels are judged ----
// Every workgroup walks a contiguous share of the buffer, eight 4 KB tiles per trip.  (Workgroups that stride over the
// whole buffer together, four loads 8 MB apart per thread, read 1.23 GB at 5.3 TB/s; this form reads it at 6.7 TB/s.)
__global__ __launch_bounds__(VEC_BLOCK) void stream_read_kernel(const uint4 *src, int64_t nvec, double *part)
{
    constexpr int U = 8;
    unsigned acc = 0;
    const int64_t per = (nvec / gridDim.x) / (VEC_BLOCK * U) * (VEC_BLOCK * U);
    const uint4 *p = src + (int64_t)blockIdx.x * per + threadIdx.x;
    for (int64_t i = 0; i < per; i += VEC_BLOCK * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = p[i + u * VEC_BLOCK];
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    // what the equal shares leave over
    for (int64_t i = (int64_t)gridDim.x * per + (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < nvec;
         i += (int64_t)gridDim.x * VEC_BLOCK) {
        const uint4 a = src[i];
        acc += a.x ^ a.y ^ a.z ^ a.w;
    }
    const double r = block_sum((double)acc);
    if (threadIdx.x == 0) part[blockIdx.x] = r;
}

hipError_t launch_stream_read(const void *src, int64_t bytes, double *part, int blocks, hipStream_t st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(VEC_BLOCK), 0, st, (const uint4 *)src, bytes / 16, part);
    return hipGetLastError();
}

// ---- validation ---------------------------------------------------------------------------
__global__ void zero_int_kernel(int32_t *x) { *x = 0; }

__global__ __launch_bounds__(VEC_BLOCK) void check_range_kernel(const int32_t *v, int64_t count, int64_t lo, int64_t hi,
                                                                 int32_t *bad)
{
    int local = 0;
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < count; i += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t x = v[i];
        local += (x < lo || x >= hi);
    }
    if (local) atomicAdd(bad, local);
}

hipError_t launch_check_range(const int32_t *v, int64_t count, int64_t lo, int64_t hi, int32_t *bad, hipStream_t st)
{
    hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, bad);
    hipLaunchKernelGGL(check_range_kernel, dim3(vec_blocks(count)), dim3(VEC_BLOCK), 0, st, v, count, lo, hi, bad);
    return hipGetLastError();
}

__global__ __launch_bounds__(VEC_BLOCK) void check_rowptr_kernel(const int32_t *rowptr, int64_t n, int64_t nnz,
                                                                  int32_t *bad)
{
    int local = 0;
    for (int64_t i = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; i < n; i += (int64_t)gridDim.x * VEC_BLOCK)
        local += (rowptr[i + 1] < rowptr[i]);
    if (blockIdx.x == 0 && threadIdx.x == 0) local += (rowptr[0] != 0) + ((int64_t)rowptr[n] != nnz);
    if (local) atomicAdd(bad, local);
}

hipError_t launch_check_rowptr(const int32_t *rowptr, int64_t n, int64_t nnz, int32_t *bad, hipStream_t st)
{
    hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, bad);
    hipLaunchKernelGGL(check_rowptr_kernel, dim3(vec_blocks(n)), dim3(VEC_BLOCK), 0, st, rowptr, n, nnz, bad);
    return hipGetLastError();
}

// ---- Alg. 2 on the device -------------------------------------------------------------------
// lines 1-5: p = 0, r = -g, s = r, p_best = s; partials of g.g
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_init_kernel(CgVecs v, double *gg_part, double *ss_part)
{
    const int64_t total = v.p * v.K;
    const T *G = (const T *)v.G;
    T *pv = (T *)v.pv, *r = (T *)v.r, *s = (T *)v.s, *pb = (T *)v.pbest;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        const T gv = G[o];
        pv[o] = T(0);
        r[o] = -gv;
        s[o] = -gv;
        pb[o] = -gv;
        local += (double)gv * (double)gv;
    }
    const double t = block_sum(local);
    if (threadIdx.x == 0) {
        gg_part[blockIdx.x] = t;
        if (ss_part) ss_part[blockIdx.x] = t;        // s_0 = -g: the same partials serve s.s
    }
}

hipError_t launch_cg_init(int dtype, const CgVecs &v, double *gg_part, double *ss_part, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_init_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, gg_part, ss_part);
    else
        hipLaunchKernelGGL(cg_init_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, gg_part, ss_part);
    return hipGetLastError();
}

__global__ __launch_bounds__(VEC_BLOCK) void cg_init_state_kernel(const double *gg_part, int nparts, CgSlot *slot0,
                                                                   const double *gg_full_part, int n_full)
{
    const double gg_in = sum_parts(gg_part, nparts);
    double goff = 0.0;
    if (gg_full_part) {
        goff = sum_parts(gg_full_part, n_full) - gg_in;
        if (!(goff > 0.0)) goff = 0.0;
    }
    const double gg = gg_in + goff;
    if (threadIdx.x == 0) {
        CgSlot s;
        s.goff = goff;
        s.rho = -1.0;
        s.sigma = -1.0;
        s.pi = 0.0;
        s.pibest = -1.0;
        s.rr = gg;
        s.rbest = sqrt(gg);
        s.gnorm = sqrt(gg);
        s.done = (gg == 0.0) ? 1 : 0;
        s.iters = 0;
        s.flags = 0;
        s.brk = 0;
        s.alpha = 0.0;
        s.best_cur = 0;
        s.best_pending = 0;
        s.sHs = 0.0;
        *slot0 = s;
    }
}

// lines 1-5 and the initial state in one launch of one block, for blocks small enough (dense workloads: a few
// thousand elements); saves a launch boundary, which costs as much as the kernel
template <typename T> __global__ __launch_bounds__(VEC_BLOCK) void cg_init_small_kernel(CgVecs v, CgSlot *slot0)
{
    const int64_t total = v.p * v.K;
    const T *G = (const T *)v.G;
    T *pv = (T *)v.pv, *r = (T *)v.r, *s = (T *)v.s, *pb = (T *)v.pbest;
    double local = 0.0;
    for (int64_t e = threadIdx.x; e < total; e += VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        const T gv = G[o];
        pv[o] = T(0);
        r[o] = -gv;
        s[o] = -gv;
        pb[o] = -gv;
        local += (double)gv * (double)gv;
    }
    const double gg = block_sum(local);
    if (threadIdx.x == 0) {
        slot0->rr = gg;
        slot0->rbest = sqrt(gg);
        slot0->gnorm = sqrt(gg);
        slot0->done = (gg == 0.0) ? 1 : 0;
        slot0->iters = 0;
        slot0->flags = 0;
        slot0->brk = 0;
        slot0->alpha = 0.0;
        slot0->best_cur = 0;
        slot0->best_pending = 0;
        slot0->sHs = 0.0;
        slot0->goff = 0.0;
        slot0->rho = -1.0;
        slot0->sigma = -1.0;
        slot0->pi = 0.0;
        slot0->pibest = -1.0;
    }
}

hipError_t launch_cg_init_small(int dtype, const CgVecs &v, CgSlot *slot0, hipStream_t st)
{
    if (dtype == SSN_F32) hipLaunchKernelGGL(cg_init_small_kernel<float>, dim3(1), dim3(VEC_BLOCK), 0, st, v, slot0);
    else hipLaunchKernelGGL(cg_init_small_kernel<double>, dim3(1), dim3(VEC_BLOCK), 0, st, v, slot0);
    return hipGetLastError();
}

hipError_t launch_cg_init_state(const double *gg_part, int nparts, CgSlot *slot0, hipStream_t st,
                                const double *gg_full_part, int n_full)
{
    hipLaunchKernelGGL(cg_init_state_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, gg_part, nparts, slot0, gg_full_part, n_full);
    return hipGetLastError();
}

// lines 1-5 on the columns the sample touches: row t of the vectors is row cols[t] of -g
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_init_support_kernel(CgVecs v, const T *G, int64_t ldg, const int32_t *cols,
                                                                     double *gg_part, double *ss_part)
{
    const int64_t total = v.p * v.K;
    T *pv = (T *)v.pv, *r = (T *)v.r, *s = (T *)v.s, *pb = (T *)v.pbest;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t t = e / v.K;
        const int c = (int)(e - t * v.K);
        const T gv = G[(int64_t)cols[t] * ldg + c];
        pv[e] = T(0);
        r[e] = -gv;
        s[e] = -gv;
        pb[e] = -gv;
        local += (double)gv * (double)gv;
    }
    const double sum = block_sum(local);
    if (threadIdx.x == 0) {
        gg_part[blockIdx.x] = sum;
        if (ss_part) ss_part[blockIdx.x] = sum;
    }
}

hipError_t launch_cg_init_support(int dtype, const CgVecs &v, const void *G, int64_t ldg, const int32_t *cols,
                                  double *gg_part, double *ss_part, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_init_support_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, (const float *)G, ldg, cols,
                           gg_part, ss_part);
    else
        hipLaunchKernelGGL(cg_init_support_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, (const double *)G, ldg,
                           cols, gg_part, ss_part);
    return hipGetLastError();
}

// The direction on all coordinates: pibest * g where the sample has no entry, the CG vector's rows elsewhere.
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_expand_fill_kernel(int64_t p, int K, const T *G, int64_t ldg, T *P, int64_t ldp,
                                                                    const CgSlot *fin)
{
    const double pibest = fin->pibest;
    const int64_t total = p * K;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK)
        P[off_of(e, K, ldp)] = (T)(pibest * (double)G[off_of(e, K, ldg)]);
}

// rows cols[] of P = the rows of pb; dot_part (nullable): one partial per block of <pb, rows cols[] of G>
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_expand_rows_kernel(int K, T *P, int64_t ldp, const T *pb, const int32_t *cols,
                                                                    int64_t ncols, const T *G, int64_t ldg, double *dot_part)
{
    const int64_t total = ncols * K;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t t = e / K;
        const int c = (int)(e - t * K);
        const int64_t col = cols[t];
        const T v = pb[e];
        P[col * ldp + c] = v;
        if (dot_part) local += (double)v * (double)G[col * ldg + c];
    }
    if (dot_part) {
        const double sum = block_sum(local);
        if (threadIdx.x == 0) dot_part[blockIdx.x] = sum;
    }
}

hipError_t launch_cg_expand(int dtype, int64_t p, int K, const void *G, int64_t ldg, void *P_out, int64_t ldp,
                            const CgSlot *fin, const void *pb, const int32_t *cols, int64_t ncols, double *dot_part,
                            int *n_dot, hipStream_t st)
{
    const int b1 = vec_blocks(p * K) * 4 > 4096 ? 4096 : vec_blocks(p * K) * 4;
    const int b2 = vec_blocks(ncols * K);                  // <= RED_MAX_PARTS: one partial per block
    if (n_dot) *n_dot = b2;
    if (dtype == SSN_F32) {
        hipLaunchKernelGGL(cg_expand_fill_kernel<float>, dim3(b1), dim3(VEC_BLOCK), 0, st, p, K, (const float *)G, ldg,
                           (float *)P_out, ldp, fin);
        hipLaunchKernelGGL(cg_expand_rows_kernel<float>, dim3(b2), dim3(VEC_BLOCK), 0, st, K, (float *)P_out, ldp,
                           (const float *)pb, cols, ncols, (const float *)G, ldg, dot_part);
    } else {
        hipLaunchKernelGGL(cg_expand_fill_kernel<double>, dim3(b1), dim3(VEC_BLOCK), 0, st, p, K, (const double *)G, ldg,
                           (double *)P_out, ldp, fin);
        hipLaunchKernelGGL(cg_expand_rows_kernel<double>, dim3(b2), dim3(VEC_BLOCK), 0, st, K, (double *)P_out, ldp,
                           (const double *)pb, cols, ncols, (const double *)G, ldg, dot_part);
    }
    return hipGetLastError();
}

// CSR path, lines 10-12: best-iterate memory, theta test, new search direction (and, with update_p, line 8)
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_step2_kernel(CgVecs v, const CgSlot *cur, CgSlot *next,
                                                              const double *rr_part, int n_rr, double theta,
                                                              double *trace_k, double *ss_part, bool update_p, double lambda)
{
    // the first element of every thread is fetched before anything waits: on small blocks that is the only
    // one, and the kernel is then two dependent round trips instead of three
    const int64_t total = v.p * v.K;
    const int64_t stride = (int64_t)gridDim.x * VEC_BLOCK;
    const int64_t e0 = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x;
    T *pw = (T *)v.pv, *s = (T *)v.s, *pb = (T *)v.pbest;
    const T *r = (const T *)v.r;
    const int64_t o0 = off_of(e0 < total ? e0 : 0, v.K, v.ld);
    T p0 = pw[o0], r0 = r[o0], s0 = s[o0];
    const CgSlot c = *cur;
    if (c.done || c.brk) {
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            CgSlot n = c;
            if (c.brk && !c.done) { n.flags |= 2; n.iters = c.iters + 1; }
            n.done = 1;
            n.brk = 0;
            *next = n;
        }
        return;
    }
    // coordinates outside the sample's columns (goff > 0 on the CSR path only): r_j = rho g_j there
    const double rho_n = c.rho - c.alpha * lambda * c.sigma;
    const double pi_n = c.pi + c.alpha * c.sigma;
    const double rr_new = sum_parts(rr_part, n_rr) + rho_n * rho_n * c.goff;
    const double rnorm = sqrt(rr_new);
    const bool better = rnorm <= c.rbest;
    const bool stop = rnorm <= theta * c.gnorm;
    const double b = rr_new / c.rr;
    double ss = 0.0;
    // one element: lines 8 (where it was left to this pass), 10 and 12
    auto element = [&](int64_t o, T pe, T re, T se) {
        T pn = pe;
        if (update_p) {                      // p += alpha s with the old s
            pn = (T)((double)pe + c.alpha * (double)se);
            pw[o] = pn;
            // lazy best-iterate memory: a better iterate is only marked; the copy happens when the next
            // iterate is worse (then the best one is the p this pass has just read) or at the very end
            if (!better && c.best_cur) pb[o] = pe;
        } else if (better) {
            pb[o] = pn;
        }
        if (!stop) {
            const T sn = (T)((double)re + b * (double)se);
            s[o] = sn;
            ss += (double)sn * (double)sn;
        }
    };
    if (update_p || better || !stop) {
        if (e0 < total) element(o0, p0, r0, s0);
        // the rest of a large block: four elements per thread in flight at a time
        constexpr int SB = 4;
        for (int64_t e = e0 + stride; e < total; e += SB * stride) {
            int64_t o[SB];
            T pe[SB], re[SB], se[SB];
#pragma unroll
            for (int u = 0; u < SB; ++u) {
                const int64_t eu = e + u * stride;
                o[u] = off_of(eu < total ? eu : e, v.K, v.ld);
                pe[u] = pw[o[u]];
                re[u] = r[o[u]];
                se[u] = s[o[u]];
            }
#pragma unroll
            for (int u = 0; u < SB; ++u)
                if (e + u * stride < total) element(o[u], pe[u], re[u], se[u]);
        }
    }
    if (ss_part) {                           // partials of s.s for the next product's curvature
        ss = block_sum(ss);
        if (threadIdx.x == 0) ss_part[blockIdx.x] = ss;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        CgSlot n;
        n.rr = rr_new;
        n.rbest = better ? rnorm : c.rbest;
        n.gnorm = c.gnorm;
        n.done = stop ? 1 : 0;
        n.iters = c.iters + 1;
        n.flags = c.flags | (stop ? 1 : 0);
        n.brk = 0;
        n.alpha = 0.0;
        n.best_cur = update_p ? (better ? 1 : 0) : 0;
        n.best_pending = 0;
        n.sHs = 0.0;
        n.goff = c.goff;
        n.rho = rho_n;
        n.pi = pi_n;
        n.pibest = better ? pi_n : c.pibest;
        n.sigma = stop ? c.sigma : rho_n + b * c.sigma;
        *next = n;
        if (trace_k) trace_k[1] = rnorm;
    }
}

hipError_t launch_cg_step2(int dtype, const CgVecs &v, const CgSlot *cur, CgSlot *next, const double *rr_part, int n_rr,
                           double theta, double *trace_k, double *ss_part, bool update_p, int blocks, hipStream_t st,
                           double lambda)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_step2_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, cur, next, rr_part, n_rr, theta,
                           trace_k, ss_part, update_p, lambda);
    else
        hipLaunchKernelGGL(cg_step2_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, cur, next, rr_part, n_rr,
                           theta, trace_k, ss_part, update_p, lambda);
    return hipGetLastError();
}

template <typename T> __global__ __launch_bounds__(VEC_BLOCK) void cg_finish_kernel(CgVecs v, const CgSlot *fin)
{
    if (!fin->best_cur) return;
    const int64_t total = v.p * v.K;
    const T *pw = (const T *)v.pv;
    T *pb = (T *)v.pbest;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        pb[o] = pw[o];
    }
}

hipError_t launch_cg_finish(int dtype, const CgVecs &v, const CgSlot *fin, int blocks, hipStream_t st)
{
    if (dtype == SSN_F32) hipLaunchKernelGGL(cg_finish_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, fin);
    else hipLaunchKernelGGL(cg_finish_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, fin);
    return hipGetLastError();
}

__global__ __launch_bounds__(VEC_BLOCK) void cg_alpha_kernel(CgSlot *cur, const double *zu_part, int n_zu,
                                                              const double *ss_part, int n_ss, double scale, double lambda,
                                                              double *trace_k)
{
    const CgSlot c = *cur;
    if (c.done) return;
    const double zu = sum_parts(zu_part, n_zu);
    const double ss = sum_parts(ss_part, n_ss) + c.sigma * c.sigma * c.goff;
    const double sHs = scale * zu + lambda * ss;
    if (threadIdx.x != 0) return;
    if (!(sHs > 0.0)) {                      // not positive definite in floating point: stop, keep p_best
        cur->brk = 1;
        if (trace_k) { trace_k[0] = 0.0; trace_k[1] = sqrt(c.rr); trace_k[2] = sHs; }
    } else {
        cur->alpha = c.rr / sHs;
        if (trace_k) { trace_k[0] = c.rr / sHs; trace_k[2] = sHs; }
    }
}

hipError_t launch_cg_alpha(CgSlot *cur, const double *zu_part, int n_zu, const double *ss_part, int n_ss, double scale,
                           double lambda, double *trace_k, hipStream_t st)
{
    hipLaunchKernelGGL(cg_alpha_kernel, dim3(1), dim3(VEC_BLOCK), 0, st, cur, zu_part, n_zu, ss_part, n_ss, scale, lambda,
                       trace_k);
    return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void cg_r_update_kernel(CgVecs v, const CgSlot *cur, double lambda, double *rr_part)
{
    const CgSlot c = *cur;
    if (c.done || c.brk) return;
    const double coef = c.alpha * lambda;
    const int64_t total = v.p * v.K;
    T *r = (T *)v.r;
    const T *s = (const T *)v.s;
    double local = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; e < total; e += (int64_t)gridDim.x * VEC_BLOCK) {
        const int64_t o = off_of(e, v.K, v.ld);
        const T rn = (T)((double)r[o] - coef * (double)s[o]);
        r[o] = rn;
        local += (double)rn * (double)rn;
    }
    const double t = block_sum(local);
    if (threadIdx.x == 0) rr_part[blockIdx.x] = t;
}

hipError_t launch_cg_r_update(int dtype, const CgVecs &v, const CgSlot *cur, double lambda, double *rr_part, int blocks,
                              hipStream_t st)
{
    if (dtype == SSN_F32)
        hipLaunchKernelGGL(cg_r_update_kernel<float>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, cur, lambda, rr_part);
    else
        hipLaunchKernelGGL(cg_r_update_kernel<double>, dim3(blocks), dim3(VEC_BLOCK), 0, st, v, cur, lambda, rr_part);
    return hipGetLastError();
}

}  // namespace ssn
