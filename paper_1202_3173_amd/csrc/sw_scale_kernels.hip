// Diagonal scaling around the product (Section 6.1): D1 C D3 = (D1 A D2) (D2^-1 B D3) with diagonal D1, D2,
// D3, chosen here as powers of two so that scaling and unscaling are exact:
//   outside scaling  D1_ii = 2^-e(max_j |A_ij|),  D3_jj = 2^-e(max_i |B_ij|)      (e = binary exponent)
//                    every row of A and every column of B gets a largest entry in [1, 2), which is what
//                    turns the norm-wise bound of a fast algorithm into one relative to ||A(i,:)|| ||B(:,j)||;
//   inside scaling   D2_kk = 2^round((e(max_j |B_kj| D3_jj) - e(max_i D1_ii |A_ik|)) / 2)
//                    column k of the scaled A and row k of the scaled B get largest entries of equal size.
// The kernels: weighted row / column maxima of |X|, the scale vectors from the maxima, and the scaled copy
// Y_ij = r_i X_ij c_j (also used in place to unscale C).  All streaming, one pass each.
#include "sw_internal.h"

namespace sw {
namespace {

constexpr int NT = 256;

// out[i] = max_j w[j] |X[i][j]|  (w == nullptr: 1).  One workgroup per row.
__global__ void __launch_bounds__(NT)
absmax_rows_kernel(const double* __restrict__ X, int64_t ld, int n, const double* __restrict__ w, double* __restrict__ out)
{
    __shared__ double red[NT / 64];
    const double* row = X + (int64_t)blockIdx.x * ld;
    double m = 0.0;
    for (int j = threadIdx.x; j < n; j += NT) {
        const double v = fabs(row[j]) * (w ? w[j] : 1.0);
        m = v > m ? v : m;           // NaN never wins: a row with NaN keeps the maximum of its numbers
    }
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_down(m, off);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < NT / 64; ++k) m = red[k] > m ? red[k] : m;
        out[blockIdx.x] = m;
    }
}

// out[j] = max(out[j], max over the workgroup's rows of w[i] |X[i][j]|); out must start at 0.  Non-negative
// doubles order like their bit patterns, so the maximum is an integer atomic on the bits.
__global__ void __launch_bounds__(NT)
absmax_cols_kernel(const double* __restrict__ X, int64_t ld, int n, const double* __restrict__ w,
                   unsigned long long* __restrict__ out, int rows_per_block)
{
    const int j = blockIdx.x * NT + threadIdx.x;
    if (j >= n) return;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(n, r0 + rows_per_block);
    double m = 0.0;
    for (int i = r0; i < r1; ++i) {
        const double v = fabs(X[(int64_t)i * ld + j]) * (w ? w[i] : 1.0);
        m = v > m ? v : m;
    }
    atomicMax(out + j, (unsigned long long)__double_as_longlong(m));
}

__device__ __forceinline__ int exponent_of(double m)
{
    // binary exponent e with 2^e <= m < 2^(e+1); zero, infinities and NaN scale by 1
    return (m > 0.0 && m < __longlong_as_double(0x7ff0000000000000LL)) ? ilogb(m) : 0;
}

__global__ void __launch_bounds__(NT)
zero_kernel(double* __restrict__ p, int n)
{
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

// s[i] = 2^-e(m[i])
__global__ void __launch_bounds__(NT)
outside_scale_kernel(const double* __restrict__ m, int n, double* __restrict__ s)
{
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i < n) s[i] = scalbn(1.0, -exponent_of(m[i]));
}

// d[k] = 2^round((e(b[k]) - e(a[k])) / 2), dinv[k] = 1 / d[k]; a column or row that is entirely zero scales by 1
__global__ void __launch_bounds__(NT)
inside_scale_kernel(const double* __restrict__ a, const double* __restrict__ b, int n, double* __restrict__ d,
                    double* __restrict__ dinv)
{
    const int k = blockIdx.x * NT + threadIdx.x;
    if (k >= n) return;
    int e = 0;
    if (a[k] > 0.0 && b[k] > 0.0) {
        const int diff = exponent_of(b[k]) - exponent_of(a[k]);
        e = (diff >= 0 ? diff + 1 : diff - 1) / 2;      // round half away from zero
    }
    d[k] = scalbn(1.0, e);
    dinv[k] = scalbn(1.0, -e);
}

// Y[i][j] = r[i] * X[i][j] * c[j]   (r or c == nullptr: 1).  Y may be X itself.
__global__ void __launch_bounds__(NT)
scale_copy_kernel(const double* X, int64_t xld, int n, const double* __restrict__ r, const double* __restrict__ c,
                  double* Y, int64_t yld)
{
    const int j = blockIdx.x * NT + threadIdx.x;
    if (j >= n) return;
    const double cj = c ? c[j] : 1.0;
    const int r0 = blockIdx.y * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int i = r0 + k;
        if (i < n) Y[(int64_t)i * yld + j] = (r ? r[i] : 1.0) * X[(int64_t)i * xld + j] * cj;
    }
}

}  // namespace

hipError_t launch_absmax_rows(const double* X, int64_t ld, int64_t n, const double* w, double* out, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(absmax_rows_kernel, dim3((unsigned)n), dim3(NT), 0, s, X, ld, (int)n, w, out);
    return hipGetLastError();
}

hipError_t launch_absmax_cols(const double* X, int64_t ld, int64_t n, const double* w, double* out, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    // cleared by a kernel, not a memset node, so that a caller may capture the call in a HIP graph
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n + NT - 1) / NT)), dim3(NT), 0, s, out, (int)n);
    const int rows_per_block = 64;
    const dim3 g((unsigned)((n + NT - 1) / NT), (unsigned)((n + rows_per_block - 1) / rows_per_block));
    hipLaunchKernelGGL(absmax_cols_kernel, g, dim3(NT), 0, s, X, ld, (int)n, w,
                       reinterpret_cast<unsigned long long*>(out), rows_per_block);
    return hipGetLastError();
}

hipError_t launch_outside_scale(const double* m, int64_t n, double* sc, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(outside_scale_kernel, dim3((unsigned)((n + NT - 1) / NT)), dim3(NT), 0, s, m, (int)n, sc);
    return hipGetLastError();
}

hipError_t launch_inside_scale(const double* a, const double* b, int64_t n, double* d, double* dinv, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(inside_scale_kernel, dim3((unsigned)((n + NT - 1) / NT)), dim3(NT), 0, s, a, b, (int)n, d, dinv);
    return hipGetLastError();
}

hipError_t launch_scale_copy(const double* X, int64_t xld, int64_t n, const double* r, const double* c, double* Y,
                             int64_t yld, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const dim3 g((unsigned)((n + NT - 1) / NT), (unsigned)((n + 7) / 8));
    hipLaunchKernelGGL(scale_copy_kernel, g, dim3(NT), 0, s, X, xld, (int)n, r, c, Y, yld);
    return hipGetLastError();
}

}  // namespace sw
