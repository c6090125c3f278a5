// Device-side generator of the seeded synthetic input matrices.
//
// Built into its own library (libsw_inputs.so); it is not part of the
// Strassen-Winograd library and contains none of the method's arithmetic.
// The entry definition is the one stated in inputs.py: a splitmix64-style
// counter hash of (seed, matrix, row * n + col), turned into a double with
// integer operations, one exact conversion and correctly rounded fp64
// multiply / divide / add, so host and device agree bit for bit.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__global__ void __launch_bounds__(256)
fill_kernel(double* __restrict__ dst, int64_t rows, int64_t cols, int64_t n, uint64_t k0, int dist)
{
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    const int64_t total = rows * cols;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += step) {
        const int64_t r = e / cols;
        const int64_t c = e - r * cols;
        const uint64_t idx = (uint64_t)r * (uint64_t)n + (uint64_t)c;
        const uint64_t z = mix64(k0 + (idx + 1ull) * gamma);
        double v;
        if (dist == 2) {
            const uint64_t k = ((z >> 32) * 17ull) >> 32;
            v = (double)(int64_t)k - 8.0;
        } else {
            const double u = (double)(z >> 11) * 0x1.0p-53;
            v = 2.0 * u - 1.0;
            if (dist == 1) v = v * (1.0 + (double)r / (double)n);
        }
        dst[r * n + c] = v;
    }
}

}  // namespace

// dst: DEVICE pointer to an n x n row-major fp64 matrix (ld = n) of which the
// leading rows x cols block is written.  stream: hipStream_t.  Returns the
// hipError_t of the launch (0 = success).  Asynchronous.
extern "C" int sw_inputs_fill(void* dst, int64_t rows, int64_t cols, int64_t n, int64_t seed,
                              int which, int dist, void* stream)
{
    if (!dst || rows < 0 || cols < 0 || rows > n || cols > n || dist < 0 || dist > 2)
        return (int)hipErrorInvalidValue;
    if (rows == 0 || cols == 0) return 0;
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    uint64_t key = 2ull * (uint64_t)seed + (uint64_t)which;
    uint64_t z = key + gamma;
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    const int64_t total = rows * cols;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (double*)dst, rows, cols, n, z, dist);
    return (int)hipGetLastError();
}
