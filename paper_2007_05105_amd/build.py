"""Build libadascale.so (HIP, gfx950) in-tree with hipcc.

The fused kernel's instances are compiled in one translation unit per register-slot level and
gain variant
(csrc/fused_level.hip with -DADASCALE_LEVEL=n -DADASCALE_LAG=0|1) beside the unit with the host code and the other
kernels (csrc/adascale.hip); the units are compiled in parallel and linked into one library.
"""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadascale.so")
LEVELS = 4

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wextra", "-Wno-unused-function", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory(prefix="adascale_build_") as tmp:
        units = [(os.path.join(CSRC, "adascale.hip"), os.path.join(tmp, "adascale.o"), [])]
        # largest units first
        units = [(os.path.join(CSRC, "fused_level.hip"), os.path.join(tmp, f"fused_level{n}_lag{lag}.o"),
                  [f"-DADASCALE_LEVEL={n}", f"-DADASCALE_LAG={lag}"])
                 for n in reversed(range(LEVELS)) for lag in (0, 1)] + units

        def compile_unit(unit):
            src, obj, extra = unit
            subprocess.run([hipcc, *HIPCC_FLAGS, *extra, "-c", src, "-o", obj], check=True)
            return obj

        with ThreadPoolExecutor(max_workers=min(len(units), os.cpu_count() or 1, 8)) as pool:
            objs = list(pool.map(compile_unit, units))
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
