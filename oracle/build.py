"""Build the CPU oracle (test infrastructure) into oracle/libsw_oracle.so with gcc.

-ffp-contract=off keeps every multiply and add separately rounded, which is
what the oracle's leaf definition states.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sw_oracle.c")
LIB = os.path.join(HERE, "libsw_oracle.so")
SRC2 = os.path.join(HERE, "sw_bilinear_oracle.c")
LIB2 = os.path.join(HERE, "libsw_bilinear_oracle.so")


def build(force: bool = True) -> str:
    for src, lib in ((SRC, LIB), (SRC2, LIB2)):
        if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
            continue
        cmd = ["gcc", "-std=c11", "-O3", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", lib, src]
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
