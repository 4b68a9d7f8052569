"""Compile the benchmark's plain streaming kernels (copy / read / write / triad /
K-way mix) for gfx950.  They calibrate the profiler's byte counters and measure
the box's own streaming ceilings; the method's library neither contains nor
calls them."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "copy_probe.hip")
LIB = os.path.join(HERE, "libabs_probe.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wextra"]


def build_probe():
    subprocess.run(["hipcc"] + FLAGS + [SRC, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build_probe())
