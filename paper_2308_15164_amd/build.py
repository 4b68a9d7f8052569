"""Compile the HIP library for gfx950 into this package directory."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "abs_sgd.hip")]
HEADERS = [os.path.join(HERE, "csrc", "abs_kernels.hpp"), os.path.join(ROOT, "include", "abs_sgd.h")]
LIB = os.path.join(HERE, "libabs_sgd.so")
PROBE_SRC = os.path.join(HERE, "csrc", "copy_probe.hip")
PROBE_LIB = os.path.join(HERE, "libabs_probe.so")

# Contraction is off so the fixed fp32 operation order survives; packed-fp32
# instruction selection is disabled on this target.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-ffp-contract=off", "-fno-fast-math",
         # the arithmetic contract needs IEEE divide and square root and fp32 subnormals kept:
         # these are hipcc's defaults, stated here so that a changed default cannot alter results
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter"]


def build_library(force=True, extra_flags=(), out=LIB):
    if not force and os.path.exists(out):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(out) >= newest:
            return out
    cmd = (["hipcc"] + FLAGS + list(extra_flags) +
           ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")] +
           SOURCES + ["-o", out])
    subprocess.run(cmd, check=True)
    return out


def build_probe():
    """Plain copy/read/write kernels the benchmark uses for calibration only."""
    subprocess.run(["hipcc"] + FLAGS + [PROBE_SRC, "-o", PROBE_LIB], check=True)
    return PROBE_LIB


if __name__ == "__main__":
    print(build_library())
    print(build_probe())
