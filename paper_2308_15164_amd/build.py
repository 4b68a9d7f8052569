"""Compile the HIP library for gfx950 into this package directory.

The sources are a handful of translation units (the C ABI, and one unit per
kernel family) compiled side by side and linked into one shared library."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
# (source, extra defines, object name)
UNITS = [("abs_sgd.hip", [], "abs_sgd"),
         ("launch_accumulate.hip", [], "launch_accumulate"),
         ("launch_accumulate_jobs.hip", [], "launch_accumulate_jobs")] + \
        [("launch_sync.hip", [f"-DABS_RULE={r}"], f"launch_sync_rule{r}") for r in range(4)]
HEADERS = [os.path.join(CSRC, h) for h in ("abs_kernels.hpp", "abs_kernels_aux.hpp", "abs_types.hpp", "abs_host.hpp")] + \
          [os.path.join(ROOT, "include", "abs_sgd.h")]
LIB = os.path.join(HERE, "libabs_sgd.so")

# Contraction is off so the fixed fp32 operation order survives; packed-fp32
# instruction selection is disabled on this target.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-ffp-contract=off", "-fno-fast-math",
         # the arithmetic contract needs IEEE divide and square root and fp32 subnormals kept:
         # these are hipcc's defaults, stated here so that a changed default cannot alter results
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter"]


def build_library(force=True, extra_flags=(), out=LIB, jobs=None):
    sources = [os.path.join(CSRC, u[0]) for u in UNITS]
    if not force and os.path.exists(out):
        newest = max(os.path.getmtime(p) for p in sources + HEADERS)
        if os.path.getmtime(out) >= newest:
            return out
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="abs_sgd_build_") as tmp:
        def compile_unit(unit):
            src, defines, name = unit
            obj = os.path.join(tmp, name + ".o")
            subprocess.run(["hipcc"] + FLAGS + list(extra_flags) + defines + inc +
                           ["-c", os.path.join(CSRC, src), "-o", obj], check=True)
            return obj
        with ThreadPoolExecutor(max_workers=jobs or min(8, len(UNITS))) as pool:
            objs = list(pool.map(compile_unit, UNITS))
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", out], check=True)
    return out


if __name__ == "__main__":
    print(build_library())
