// The product for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): the same recursion, planner, executor and kernels as sw_gemm_ex, with the
// workspace taken from an array that is part of the library's own device image instead of a caller's buffer.
//
// Every GPU the library is loaded on holds its own copy of `scratch` at its own address for the life of the
// process.  In host code the array's NAME is only a stand-in for the symbol; the device address is asked for
// once per device (hipGetSymbolAddress, with that device current) and only that pointer is ever used.
#include <mutex>
#include <string>

#include "sw_internal.h"

namespace sw {
namespace {

static __device__ __align__(256) unsigned char scratch[SW_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};   // device address of this device's copy of `scratch`, asked for on first use

// -> the calling thread's current device's scratch pointer, or nullptr with the error text set
void* scratch_for_current_device()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { hip_fail(e, "hipGetDevice"); return nullptr; }
    if (dev < 0 || dev >= MAX_DEVICES) { set_error("device %d is beyond the %d devices the static scratch supports", dev, MAX_DEVICES); return nullptr; }
    std::lock_guard<std::mutex> g(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) { hip_fail(e, "hipGetSymbolAddress(scratch)"); return nullptr; }
        if (!p || ((uintptr_t)p & 255u)) { set_error("static scratch has no usable address on device %d", dev); return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace
}  // namespace sw

using namespace sw;

extern "C" int sw_gemm_static(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                              int levels, const char* schedule, void* hip_stream)
{
    // Every argument check, the size limit included, comes before anything touches the device.
    CallOpts opts{0, SW_ODD_PAD, false, true};   // one stream (no streams or events are created), no event brackets, zero padding
    int rc = gemm_rect_impl(Dims{n, n, n}, A, lda, B, ldb, C, ldc, levels, schedule, nullptr, (int64_t)SW_STATIC_SCRATCH_BYTES,
                            (hipStream_t)hip_stream, opts);
    if (rc == SW_ENOMEM) {
        const std::string why = sw_last_error();
        set_error("sw_gemm_static: the static scratch of %lld bytes is too small (%s); use sw_gemm_ex with a workspace of the caller's",
                  (long long)SW_STATIC_SCRATCH_BYTES, why.c_str());
    }
    if (rc != SW_OK) return rc;
    void* ws = scratch_for_current_device();
    if (!ws) return SW_EHIP;
    opts.check_only = false;
    return gemm_rect_impl(Dims{n, n, n}, A, lda, B, ldb, C, ldc, levels, schedule, ws, (int64_t)SW_STATIC_SCRATCH_BYTES,
                          (hipStream_t)hip_stream, opts);
}
