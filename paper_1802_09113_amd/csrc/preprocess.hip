// Preprocessing of Sec. 4 (unit column norms): every column of X is divided by its 2-norm, in place, on the
// device.  A set-up step (it runs once per data set, before ssn_create), kept deterministic like the rest:
// dense columns are summed per row chunk and the chunk sums added in order; CSR columns are summed through
// the same column-sorted gather as the transposed products (csc.hip) applied to the squared values.
#include "ssn_internal.h"

namespace ssn {

// part[chunk * p + j] = sum over the chunk's rows of X[i][j]^2 ; one thread per column, rows in order
template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void colsq_part_kernel(const T *X, int64_t ldx, int64_t n, int64_t p,
                                                                int64_t rows_per_chunk, double *part)
{
    const int64_t j = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x;
    if (j >= p) return;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
    const int64_t r1 = (r0 + rows_per_chunk < n) ? r0 + rows_per_chunk : n;
    double s = 0.0;
    for (int64_t i = r0; i < r1; ++i) {
        const double x = (double)X[i * ldx + j];
        s += x * x;
    }
    part[(int64_t)blockIdx.y * p + j] = s;
}

__global__ __launch_bounds__(VEC_BLOCK) void colsq_reduce_kernel(const double *part, int nchunks, int64_t p, double *colnorm)
{
    const int64_t j = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x;
    if (j >= p) return;
    double s = 0.0;
    for (int c = 0; c < nchunks; ++c) s += part[(int64_t)c * p + j];
    colnorm[j] = sqrt(s);
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void dense_scale_kernel(T *X, int64_t ldx, int64_t n, int64_t p, const double *colnorm)
{
    const int64_t j = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x;
    if (j >= p) return;
    const double cn = colnorm[j];
    if (!(cn > 0.0)) return;
    for (int64_t i = blockIdx.y; i < n; i += gridDim.y) X[i * ldx + j] = (T)((double)X[i * ldx + j] / cn);
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void square_kernel(const T *v, int64_t nnz, T *sq)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK)
        sq[t] = v[t] * v[t];
}

template <typename T> __global__ __launch_bounds__(VEC_BLOCK) void fill_kernel(T *v, int64_t count, T value)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < count; t += (int64_t)gridDim.x * VEC_BLOCK)
        v[t] = value;
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void sqrt_to_double_kernel(const T *ss, int64_t p, double *colnorm)
{
    for (int64_t j = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; j < p; j += (int64_t)gridDim.x * VEC_BLOCK)
        colnorm[j] = sqrt((double)ss[j]);
}

template <typename T>
__global__ __launch_bounds__(VEC_BLOCK) void csr_scale_kernel(T *vals, const int32_t *colidx, int64_t nnz, const double *colnorm)
{
    for (int64_t t = (int64_t)blockIdx.x * VEC_BLOCK + threadIdx.x; t < nnz; t += (int64_t)gridDim.x * VEC_BLOCK) {
        const double cn = colnorm[colidx[t]];
        if (cn > 0.0) vals[t] = (T)((double)vals[t] / cn);
    }
}

static unsigned blocks_for(int64_t n)
{
    int64_t b = (n + VEC_BLOCK - 1) / VEC_BLOCK;
    if (b > 16384) b = 16384;
    if (b < 1) b = 1;
    return (unsigned)b;
}

#define PRE_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) {                         \
            cleanup();                                  \
            return e_;                                  \
        }                                               \
    } while (0)

template <typename T>
static hipError_t normalize_dense(T *X, int64_t ldx, int64_t n, int64_t p, double *colnorm, hipStream_t st)
{
    double *part = nullptr;
    auto cleanup = [&]() {
        if (part) (void)hipFree(part);
    };
    const int64_t ctiles = (p + VEC_BLOCK - 1) / VEC_BLOCK;
    int64_t nchunks = (2048 + ctiles - 1) / ctiles;              // about 2048 blocks in all
    if (nchunks > (n + 63) / 64) nchunks = (n + 63) / 64;        // at least 64 rows per chunk
    if (nchunks > 65535) nchunks = 65535;
    if (nchunks < 1) nchunks = 1;
    const int64_t rpc = (n + nchunks - 1) / nchunks;
    nchunks = (n + rpc - 1) / rpc;
    PRE_HIP(hipMalloc((void **)&part, sizeof(double) * (size_t)nchunks * (size_t)p));
    hipLaunchKernelGGL(colsq_part_kernel<T>, dim3((unsigned)ctiles, (unsigned)nchunks), dim3(VEC_BLOCK), 0, st, X, ldx, n, p,
                       rpc, part);
    hipLaunchKernelGGL(colsq_reduce_kernel, dim3((unsigned)ctiles), dim3(VEC_BLOCK), 0, st, part, (int)nchunks, p, colnorm);
    int64_t ry = n < 1024 ? n : 1024;
    hipLaunchKernelGGL(dense_scale_kernel<T>, dim3((unsigned)ctiles, (unsigned)ry), dim3(VEC_BLOCK), 0, st, X, ldx, n, p,
                       colnorm);
    PRE_HIP(hipGetLastError());
    PRE_HIP(hipStreamSynchronize(st));
    cleanup();
    return hipSuccess;
}

template <typename T>
static hipError_t normalize_csr(int dtype, const int32_t *rowptr, const int32_t *colidx, T *vals, int64_t n, int64_t p,
                                int64_t nnz, double *colnorm, hipStream_t st)
{
    T *sq = nullptr, *ones = nullptr, *ss = nullptr;
    CscView view;
    auto cleanup = [&]() {
        if (sq) (void)hipFree(sq);
        if (ones) (void)hipFree(ones);
        if (ss) (void)hipFree(ss);
        csc_free(&view);
    };
    PRE_HIP(hipMalloc((void **)&ss, sizeof(T) * (size_t)p));
    hipLaunchKernelGGL(fill_kernel<T>, dim3(blocks_for(p)), dim3(VEC_BLOCK), 0, st, ss, p, T(0));
    if (nnz > 0) {
        PRE_HIP(hipMalloc((void **)&sq, sizeof(T) * (size_t)nnz));
        PRE_HIP(hipMalloc((void **)&ones, sizeof(T) * (size_t)n));
        hipLaunchKernelGGL(square_kernel<T>, dim3(blocks_for(nnz)), dim3(VEC_BLOCK), 0, st, vals, nnz, sq);
        hipLaunchKernelGGL(fill_kernel<T>, dim3(blocks_for(n)), dim3(VEC_BLOCK), 0, st, ones, n, T(1));
        // column sums of the squared values = X2^T * 1 on the column-sorted view of all rows
        PRE_HIP(csc_build(&view, dtype, rowptr, colidx, sq, nullptr, n, p, 1, st));
        PRE_HIP(launch_csc_apply(dtype, view, 1, 1, ones, 1.0, ss, 1, nullptr, nullptr, st));
    }
    hipLaunchKernelGGL(sqrt_to_double_kernel<T>, dim3(blocks_for(p)), dim3(VEC_BLOCK), 0, st, ss, p, colnorm);
    if (nnz > 0)
        hipLaunchKernelGGL(csr_scale_kernel<T>, dim3(blocks_for(nnz)), dim3(VEC_BLOCK), 0, st, vals, colidx, nnz, colnorm);
    PRE_HIP(hipGetLastError());
    PRE_HIP(hipStreamSynchronize(st));
    cleanup();
    return hipSuccess;
}

hipError_t normalize_columns(int layout, int dtype, int64_t n, int64_t p, void *X, int64_t ldx, const int32_t *rowptr,
                             const int32_t *colidx, void *vals, int64_t nnz, double *colnorm, hipStream_t st)
{
    if (layout == SSN_DENSE_ROWMAJOR) {
        return dtype == SSN_F32 ? normalize_dense<float>((float *)X, ldx, n, p, colnorm, st)
                                : normalize_dense<double>((double *)X, ldx, n, p, colnorm, st);
    }
    return dtype == SSN_F32 ? normalize_csr<float>(dtype, rowptr, colidx, (float *)vals, n, p, nnz, colnorm, st)
                            : normalize_csr<double>(dtype, rowptr, colidx, (double *)vals, n, p, nnz, colnorm, st);
}

}  // namespace ssn
