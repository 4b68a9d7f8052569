"""Builds tests/c_abi/abi_check: a plain C99 program (gcc, no HIP compiler) that
calls the C ABI with hipMalloc'ed memory and compares against the C oracle.
TEST INFRASTRUCTURE: links liboracle.so; nothing in the product uses it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "abi_check.c")
EXE = os.path.join(HERE, "abi_check")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_abi_check(force=False):
    """Needs libabs_sgd.so and liboracle.so to be built already."""
    deps = [SRC, os.path.join(ROOT, "include", "abs_sgd.h")]
    if not force and os.path.exists(EXE) and all(os.path.getmtime(EXE) >= os.path.getmtime(d) for d in deps):
        return EXE
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-O1",
           "-D__HIP_PLATFORM_AMD__",                    # selects the AMD side of the HIP runtime header
           "-I", os.path.join(ROCM, "include"), "-I", os.path.join(ROOT, "include"), SRC, "-o", EXE,
           "-L", os.path.join(ROOT, "paper_2308_15164_amd"), "-labs_sgd",
           "-L", os.path.join(ROOT, "oracle"), "-loracle",
           "-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2308_15164_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    subprocess.run(cmd, check=True)
    return EXE


if __name__ == "__main__":
    print(build_abi_check(force=True))
