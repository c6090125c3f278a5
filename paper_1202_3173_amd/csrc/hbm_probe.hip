// Measurement only (its own library, libsw_probe.so; nothing in the product links or loads it): synthetic
// streaming kernels with NIN input streams and NOUT output streams of equal length, 16 bytes per lane per
// access, one pass, non-temporal hints -- the access pattern of the addition kernels without their arithmetic
// detail.  kernel_bench's `streams` command sweeps (NIN, NOUT) to show how the rate HBM sustains depends on the
// number of streams a kernel reads and writes at once; that sweep is the ceiling the addition kernels are
// measured against.  Its `beside` command runs the leaf products next to background traffic of a chosen number of
// workgroups (load_kernel) and reads the shader clock meanwhile (meter_kernel).
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace {

typedef double v2d __attribute__((ext_vector_type(2)));

// every output is the sum of ALL inputs plus one of them (or a constant when there is no input), so no load can
// be dropped; every input is read once; with no output the sum of the inputs is kept alive by a store that never
// happens (guard is false at run time).  A workgroup works on CH consecutive pieces of 256 lanes x 16 bytes of
// every stream per trip and writes stream by stream (CH pieces of one output, then the next output), so CH > 1
// shows whether longer contiguous spans per stream and workgroup change what HBM sustains.
template <int NIN, int NOUT, int CH>
__global__ void __launch_bounds__(256) streams_kernel(const v2d* __restrict__ in, v2d* __restrict__ out, int64_t n2,
                                                      int64_t in_stride, int64_t out_stride, int guard)
{
    constexpr int64_t SPAN = 256 * CH;
    for (int64_t base = (int64_t)blockIdx.x * SPAN + threadIdx.x; base < n2; base += (int64_t)gridDim.x * SPAN) {
        v2d s[CH], x[CH][NIN > 0 ? NIN : 1];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int64_t i = base + c * 256;
#pragma unroll
            for (int k = 0; k < (NIN > 0 ? NIN : 1); ++k) x[c][k] = (v2d){1.0, 2.0};
            if (i < n2) {
#pragma unroll
                for (int k = 0; k < NIN; ++k) x[c][k] = __builtin_nontemporal_load(in + k * in_stride + i);
            }
            s[c] = x[c][0];
#pragma unroll
            for (int k = 1; k < NIN; ++k) s[c] += x[c][k];
            if (NOUT == 0 && guard && i < n2 && s[c][0] == 0.12345) out[i] = s[c];
        }
#pragma unroll
        for (int j = 0; j < NOUT; ++j) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int64_t i = base + c * 256;
                if (i < n2) __builtin_nontemporal_store(s[c] + x[c][NIN > 0 ? j % NIN : 0], out + j * out_stride + i);
            }
        }
    }
}

// Background traffic for the `beside` measurement: `reps` passes over n2 elements of 16 bytes with however many
// workgroups it is launched with.  mode 0: copy (one stream in, one out), 1: read only, 2: write only.
__global__ void __launch_bounds__(256) load_kernel(const v2d* __restrict__ in, v2d* __restrict__ out, int64_t n2, int reps, int mode,
                                                   int guard)
{
    v2d keep = (v2d){0.0, 0.0};
    for (int r = 0; r < reps; ++r) {
        for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < n2; i += (int64_t)gridDim.x * 1024) {
            v2d x[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) x[c] = mode == 2 ? (v2d){1.0 + r, 2.0} : __builtin_nontemporal_load(in + i + c * 256);
            if (mode == 1) {
#pragma unroll
                for (int c = 0; c < 4; ++c) keep += x[c];
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) __builtin_nontemporal_store(x[c], out + i + c * 256);
            }
        }
    }
    if (mode == 1 && guard && keep[0] == 0.12345) out[threadIdx.x] = keep;
}

// One wavefront that sleeps `iters` times about 8000 clocks and notes the shader-clock counter and the constant
// 100 MHz counter before and after: out[0..3] = clock at start, at end, 100 MHz count at start, at end.  Their
// ratio is the average shader clock while other kernels run.
__global__ void __launch_bounds__(64) meter_kernel(int64_t* out, int iters)
{
    const int64_t c0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) __builtin_amdgcn_s_sleep(127);
    const int64_t c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { out[0] = c0; out[1] = c1; out[2] = w0; out[3] = w1; }
}

// The matrix pipes alone: every wavefront issues `iters` rounds of 16 independent v_mfma_f64_16x16x4_f64 on operands
// held in registers (the accumulator tile of the leaf kernel, 4 x 4 MFMA tiles, without its loads).  Two workgroups of
// four wavefronts per CU, as the leaf kernel runs.  2 * 16 * 16 * 4 = 2048 flops per instruction and wavefront.
typedef double v4d __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256, 2) mfma_kernel(double* __restrict__ out, int iters, double a0, double b0)
{
    v4d acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = (v4d){0.0, 0.0, 0.0, 0.0};
    const double a = a0 + 1e-9 * (double)(threadIdx.x & 63), b = b0;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[t], 0, 0, 0);
    }
    v4d s = acc[0];
#pragma unroll
    for (int t = 1; t < 16; ++t) s += acc[t];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = (s[0] + s[1]) + (s[2] + s[3]);
}

}  // namespace

// n2: elements of 16 bytes per stream; chunks: 1, or 4 for (1, 8), (4, 7), (7, 4) and (16, 49) streams;
// blocks: workgroups of 256 threads (grid-stride).  Returns 0, -1 for a combination that is not instantiated, or
// the HIP error code.
extern "C" int sw_probe_streams(int nin, int nout, int chunks, const void* in, void* out, int64_t n2, int64_t in_stride,
                                int64_t out_stride, int blocks, void* hip_stream)
{
    hipStream_t s = (hipStream_t)hip_stream;
    if (blocks < 1 || n2 < 0) return -1;
#define SW_CASE(I, O, CH)                                                                                                     \
    if (nin == I && nout == O && chunks == CH) {                                                                              \
        hipLaunchKernelGGL((streams_kernel<I, O, CH>), dim3(blocks), dim3(256), 0, s, (const v2d*)in, (v2d*)out, n2,          \
                           in_stride, out_stride, 0);                                                                         \
        return (int)hipGetLastError();                                                                                        \
    }
    SW_CASE(0, 1, 1) SW_CASE(1, 0, 1) SW_CASE(1, 1, 1) SW_CASE(2, 1, 1) SW_CASE(1, 4, 1) SW_CASE(1, 8, 1) SW_CASE(4, 1, 1)
    SW_CASE(4, 4, 1) SW_CASE(4, 7, 1) SW_CASE(7, 4, 1) SW_CASE(5, 3, 1) SW_CASE(16, 49, 1) SW_CASE(49, 16, 1) SW_CASE(8, 8, 1)
    SW_CASE(16, 16, 1)
    SW_CASE(1, 8, 4) SW_CASE(4, 7, 4) SW_CASE(7, 4, 4) SW_CASE(16, 49, 4)
#undef SW_CASE
    return -1;
}

// Background traffic (see load_kernel): in / out hold n2 elements of 16 bytes each (n2 >= 1024).  Returns 0, -1 for
// arguments out of range, or the HIP error code.
extern "C" int sw_probe_load(const void* in, void* out, int64_t n2, int reps, int mode, int blocks, void* hip_stream)
{
    if (blocks < 1 || n2 < 1024 || reps < 0 || mode < 0 || mode > 2) return -1;
    hipLaunchKernelGGL(load_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, (const v2d*)in, (v2d*)out, n2, reps, mode, 0);
    return (int)hipGetLastError();
}

// The clock meter (see meter_kernel): out holds four int64.
extern "C" int sw_probe_meter(void* out, int iters, void* hip_stream)
{
    if (iters < 0) return -1;
    hipLaunchKernelGGL(meter_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, (int64_t*)out, iters);
    return (int)hipGetLastError();
}

// The matrix-pipe probe (see mfma_kernel): out holds blocks * 256 doubles.  Returns 0, -1, or the HIP error code.
extern "C" int sw_probe_mfma(void* out, int blocks, int iters, void* hip_stream)
{
    if (blocks < 1 || iters < 0) return -1;
    hipLaunchKernelGGL(mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, (double*)out, iters, 1.0, 0.5);
    return (int)hipGetLastError();
}
