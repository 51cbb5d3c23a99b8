"""Builds the package's native libraries in-tree with hipcc for gfx950.

    python -m paper_2505_09764_amd.build

Two shared objects are produced next to this file:
  libfast.so            the synthesis library (C ABI of include/fast.h)
  libfast_workloads.so  the synthetic traffic generator (input data only)
"""
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_INC = os.path.join(os.path.dirname(_HERE), "include")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops is switched off on purpose: packed FP32 forms have produced
# silently wrong results on the target machines.
COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]

LIB_FAST = os.path.join(_HERE, "libfast.so")
LIB_WORKLOADS = os.path.join(_HERE, "libfast_workloads.so")

# The synthesis library: source file -> extra compiler flags.  The decomposition kernels'
# stage loops are chains of dependent instructions run by one wavefront per matrix; the
# scheduler strategy that maximises instruction-level parallelism shortens them (cfg5: k2
# 11.68 -> 11.37 ms, k9 76 -> 71 ms) but slows the redistribution kernels by 15 %, so it is
# applied to that translation unit only.
FAST_SOURCES = {
    "fast_api.hip": [],
    "decompose.hip": ["-mllvm", "-amdgpu-sched-strategy=max-ilp"],
}
WORKLOAD_SOURCES = {"workload_gen.hip": []}

_OBJ_FLAGS = [f for f in COMMON_FLAGS if f != "-shared"]


def _compile(out, sources):
    """Compiles every source to an object with its own flags, then links the shared object."""
    objs = []
    for src, extra in sources.items():
        obj = os.path.join(_HERE, "_build", os.path.splitext(src)[0] + ".o")
        os.makedirs(os.path.dirname(obj), exist_ok=True)
        subprocess.check_call([HIPCC] + _OBJ_FLAGS + ["-I", _INC, "-I", _CSRC] + extra +
                              ["-c", "-o", obj, os.path.join(_CSRC, src)])
        objs.append(obj)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC",
                           "-Wno-unused-command-line-argument", "-o", out] + objs)
    return out


def build_fast():
    return _compile(LIB_FAST, FAST_SOURCES)


def build_workloads():
    return _compile(LIB_WORKLOADS, WORKLOAD_SOURCES)


def build_all():
    build_fast()
    build_workloads()


if __name__ == "__main__":
    build_all()
    print("built", LIB_FAST, LIB_WORKLOADS, file=sys.stderr)
