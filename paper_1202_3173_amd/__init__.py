"""MI355X-native Strassen-Winograd fp64 matrix multiply (the on-device hot path of CAPS).

`binding` holds the ctypes front end of the C ABI (include/sw_gemm.h); `inputs` the seeded synthetic
matrices used by tests and the benchmark.  Importing the package loads no native code; the first call into
`binding` does, and fails loudly if libsw_gemm.so has not been built."""
