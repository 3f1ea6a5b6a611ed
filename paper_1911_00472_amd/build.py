"""Build the gfx950 shared library (hipcc cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "pcr_lib.hip")
LIB = os.path.join(HERE, "libpcr.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build():
    """Compile csrc/ into libpcr.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC])
    return LIB


if __name__ == "__main__":
    print(build())
