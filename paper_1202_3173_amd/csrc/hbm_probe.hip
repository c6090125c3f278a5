// Measurement only (its own library, libsw_probe.so; nothing in the product links or loads it): synthetic
// streaming kernels with NIN input streams and NOUT output streams of equal length, 16 bytes per lane per
// access, one pass, non-temporal hints -- the access pattern of the addition kernels without their arithmetic
// detail.  kernel_bench's `streams` command sweeps (NIN, NOUT) to show how the rate HBM sustains depends on the
// number of streams a kernel reads and writes at once; that sweep is the ceiling the addition kernels are
// measured against.
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
