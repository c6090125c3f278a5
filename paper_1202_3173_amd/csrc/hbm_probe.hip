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
// happens (guard is false at run time)
template <int NIN, int NOUT>
__global__ void __launch_bounds__(256) streams_kernel(const v2d* __restrict__ in, v2d* __restrict__ out, int64_t n2,
                                                      int64_t in_stride, int64_t out_stride, int guard)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n2; i += (int64_t)gridDim.x * 256) {
        v2d x[NIN > 0 ? NIN : 1];
        if (NIN == 0) x[0] = (v2d){1.0, 2.0};
#pragma unroll
        for (int k = 0; k < NIN; ++k) x[k] = __builtin_nontemporal_load(in + k * in_stride + i);
        v2d s = x[0];
#pragma unroll
        for (int k = 1; k < NIN; ++k) s += x[k];
        if (NOUT == 0 && guard && s[0] == 0.12345) out[i] = s;
#pragma unroll
        for (int j = 0; j < NOUT; ++j) __builtin_nontemporal_store(s + x[NIN > 0 ? j % NIN : 0], out + j * out_stride + i);
    }
}

}  // namespace

// n2: elements of 16 bytes per stream; blocks: workgroups of 256 threads (grid-stride).  Returns 0, -1 for a
// stream count that is not instantiated, or the HIP error code.
extern "C" int sw_probe_streams(int nin, int nout, const void* in, void* out, int64_t n2, int64_t in_stride, int64_t out_stride,
                                int blocks, void* hip_stream)
{
    hipStream_t s = (hipStream_t)hip_stream;
#define SW_CASE(I, O)                                                                                                         \
    if (nin == I && nout == O) {                                                                                              \
        hipLaunchKernelGGL((streams_kernel<I, O>), dim3(blocks), dim3(256), 0, s, (const v2d*)in, (v2d*)out, n2, in_stride,   \
                           out_stride, 0);                                                                                    \
        return (int)hipGetLastError();                                                                                        \
    }
    SW_CASE(0, 1) SW_CASE(1, 0) SW_CASE(1, 1) SW_CASE(2, 1) SW_CASE(1, 4) SW_CASE(1, 8) SW_CASE(4, 1) SW_CASE(4, 4) SW_CASE(4, 7)
    SW_CASE(7, 4) SW_CASE(5, 3) SW_CASE(16, 49) SW_CASE(49, 16) SW_CASE(8, 8) SW_CASE(16, 16)
#undef SW_CASE
    return -1;
}
