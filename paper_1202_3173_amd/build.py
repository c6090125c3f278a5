"""Compile the HIP sources for gfx950 into in-tree shared libraries.

  libsw_gemm.so    the product: planner, executor, kernels, C ABI (include/sw_gemm.h)
  libsw_inputs.so  the device-side synthetic input generator (not part of the product path)
  libsw_probe.so   synthetic multi-stream copy kernels for the bandwidth sweep of kernel_bench (measurement only)

hipcc cross-compiles without a GPU.  Flags: packed-FP32 code generation is switched off (the
instructions are not trusted on the test machines); MFMA results stay in ordinary VGPRs
(-amdgpu-mfma-vgpr-form) so the accumulators of the leaf GEMM are never copied to and from AGPRs.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsw_gemm.so")
INPUTS_LIB = os.path.join(HERE, "libsw_inputs.so")
PROBE_LIB = os.path.join(HERE, "libsw_probe.so")

COMMON = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument"]
PRODUCT_SOURCES = ["sw_api.hip", "sw_add_kernels.hip", "sw_leaf_gemm.hip", "sw_scale_kernels.hip", "sw_bilinear.hip", "sw_dgemm.hip", "sw_static.hip", "sw_peel_kernels.hip"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose=False):
    out = _run(COMMON + ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                         "-o", LIB] + [os.path.join(CSRC, s) for s in PRODUCT_SOURCES])
    out += _run(COMMON + ["-ffp-contract=off", "-o", INPUTS_LIB, os.path.join(CSRC, "inputs_fill.hip")])
    out += _run(COMMON + ["-o", PROBE_LIB, os.path.join(CSRC, "hbm_probe.hip")])
    if verbose and out.strip():
        print(out)
    return LIB, INPUTS_LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
