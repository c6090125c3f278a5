// The one-wide products of a level whose odd extents are peeled (Section 3.1, "dynamic peeling"; SW_ODD_PEEL_LEVELS):
// with the last row, column and inner index of a problem C = A * B split off,
//
//     c12 = [A11 a12] * [b12; b22]        a matrix times a column        (matvec)
//     [c21 c22] = [a21 a22] * B           a row times a matrix           (vecmat)
//     C11 += a12 * b21                    a rank-one update              (rank1)
//
// Each reads its matrix once, so all three are bound by HBM; on the 128 x 128 tiles of the MFMA kernel a one-wide
// product computes 128 times what it needs.  All are batched over the `live` problems of the level (blockIdx.y or
// blockIdx.z), use 8-byte accesses only (no alignment is assumed) and add in a fixed order, so a result does not
// depend on the launch or on the step order around it.
#include "sw_internal.h"

namespace sw {
namespace {

constexpr int NT = 256;
constexpr int MV_ROWS = 16;        // rows of A per workgroup (four per wavefront, in flight together)
constexpr int MV_KC = 2048;        // elements of the column staged in LDS at a time
constexpr int VM_COLS = 64;        // columns of B per workgroup: one per lane, the four wavefronts split k
constexpr int R1_ROWS = 4;         // rows per thread of the rank-one update

// y_b[i] = sum_k A_b[i][k] * x_b[k], i < M, k < K.  x and y are columns: element k at x + k * xld.
__global__ void __launch_bounds__(NT)
matvec_kernel(const double* __restrict__ A, int64_t lda, int64_t sa, const double* __restrict__ x, int64_t xld, int64_t sx,
              double* __restrict__ y, int64_t yld, int64_t sy, int M, int K)
{
    __shared__ double xs[MV_KC];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t b = blockIdx.y;
    const double* Ab = A + b * sa;
    const double* xb = x + b * sx;
    const int row0 = blockIdx.x * MV_ROWS + wave * 4;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int k0 = 0; k0 < K; k0 += MV_KC) {
        const int kc = min(MV_KC, K - k0);
        __syncthreads();                                   // the previous chunk has been used by every wavefront
        for (int t = threadIdx.x; t < kc; t += NT) xs[t] = xb[(int64_t)(k0 + t) * xld];
        __syncthreads();
        for (int k = lane; k < kc; k += 64) {
            const double xv = xs[k];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (row0 + r < M) acc[r] += Ab[(int64_t)(row0 + r) * lda + k0 + k] * xv;
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        double v = acc[r];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0 && row0 + r < M) y[b * sy + (int64_t)(row0 + r) * yld] = v;
    }
}

// y_b[j] = sum_k x_b[k] * B_b[k][j], j < N, k < K.  x and y are rows (contiguous).
__global__ void __launch_bounds__(NT)
vecmat_kernel(const double* __restrict__ x, int64_t sx, const double* __restrict__ B, int64_t ldb, int64_t sb,
              double* __restrict__ y, int64_t sy, int N, int K)
{
    __shared__ double part[4][VM_COLS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t b = blockIdx.y;
    const double* xb = x + b * sx;
    const double* Bb = B + b * sb;
    const int j = blockIdx.x * VM_COLS + lane;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    if (j < N) {
        // wavefront w takes k = w, w + 4, ...; four independent partial sums keep four loads in flight
        int k = wave;
        for (; k + 12 < K; k += 16) {
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] += xb[k + 4 * u] * Bb[(int64_t)(k + 4 * u) * ldb + j];
        }
        for (; k < K; k += 4) acc[0] += xb[k] * Bb[(int64_t)k * ldb + j];
    }
    part[wave][lane] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    if (wave == 0 && j < N) y[b * sy + j] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

// C_b[i][j] += u_b[i] * v_b[j], i < M, j < N.  u is a column (element i at u + i * uld), v a row.
__global__ void __launch_bounds__(NT)
rank1_kernel(const double* __restrict__ u, int64_t uld, int64_t su, const double* __restrict__ v, int64_t sv,
             double* __restrict__ C, int64_t ldc, int64_t sc, int M, int N)
{
    const int j = blockIdx.x * NT + threadIdx.x;
    if (j >= N) return;
    const int64_t b = blockIdx.z;
    const int r0 = blockIdx.y * R1_ROWS;
    const double vj = v[b * sv + j];
    double* Cb = C + b * sc;
    double c[R1_ROWS], ui[R1_ROWS];
#pragma unroll
    for (int r = 0; r < R1_ROWS; ++r) {
        if (r0 + r < M) {
            c[r] = Cb[(int64_t)(r0 + r) * ldc + j];
            ui[r] = u[b * su + (int64_t)(r0 + r) * uld];
        }
    }
#pragma unroll
    for (int r = 0; r < R1_ROWS; ++r)
        if (r0 + r < M) Cb[(int64_t)(r0 + r) * ldc + j] = c[r] + ui[r] * vj;
}

inline bool grid_ok(int64_t x, int64_t y, int64_t z) { return x > 0 && x <= 0x7fffffffLL && y > 0 && y <= 65535 && z > 0 && z <= 65535; }

}  // namespace

hipError_t launch_matvec(int64_t M, int64_t K, int64_t live, Mat a, Mat x, Mat y, hipStream_t s)
{
    if (M == 0 || live == 0) return hipSuccess;
    if (K == 0) return hipErrorInvalidValue;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_GEMM, s, {fp(a, M, K, live), fp(x, K, 1, live)}, {fp(y, M, 1, live)});
    const int64_t gx = (M + MV_ROWS - 1) / MV_ROWS;
    if (!grid_ok(gx, live, 1) || M > 0x7fffffffLL || K > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(matvec_kernel, dim3((unsigned)gx, (unsigned)live), dim3(NT), 0, s, a.p, a.ld, a.stride, x.p, x.ld, x.stride, y.p,
                       y.ld, y.stride, (int)M, (int)K);
    return hipGetLastError();
}

hipError_t launch_vecmat(int64_t N, int64_t K, int64_t live, Mat x, Mat b, Mat y, hipStream_t s)
{
    if (N == 0 || live == 0) return hipSuccess;
    if (K == 0) return hipErrorInvalidValue;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_GEMM, s, {fp(x, 1, K, live), fp(b, K, N, live)}, {fp(y, 1, N, live)});
    const int64_t gx = (N + VM_COLS - 1) / VM_COLS;
    if (!grid_ok(gx, live, 1) || N > 0x7fffffffLL || K > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(vecmat_kernel, dim3((unsigned)gx, (unsigned)live), dim3(NT), 0, s, x.p, x.stride, b.p, b.ld, b.stride, y.p, y.stride,
                       (int)N, (int)K);
    return hipGetLastError();
}

hipError_t launch_rank1(int64_t M, int64_t N, int64_t live, Mat u, Mat v, Mat c, hipStream_t s)
{
    if (M == 0 || N == 0 || live == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_GEMM, s, {fp(u, M, 1, live), fp(v, 1, N, live), fp(c, M, N, live)}, {fp(c, M, N, live)});
    const int64_t gx = (N + NT - 1) / NT, gy = (M + R1_ROWS - 1) / R1_ROWS;
    if (!grid_ok(gx, gy, live) || M > 0x7fffffffLL || N > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rank1_kernel, dim3((unsigned)gx, (unsigned)gy, (unsigned)live), dim3(NT), 0, s, u.p, u.ld, u.stride, v.p, v.stride, c.p,
                       c.ld, c.stride, (int)M, (int)N);
    return hipGetLastError();
}

}  // namespace sw
