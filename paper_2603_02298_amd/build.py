"""Builds liblayoutcopy.so (host algebra + planner + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_PATH = os.path.join(HERE, "liblayoutcopy.so")
SOURCES = ["layout.cpp", "algebra.cpp", "semimodule.cpp", "plan.cpp", "replay.cpp", "capi.cpp", "kernels.hip"]
HEADERS = ["layout.hpp", "algebra.hpp", "plan.hpp", "kernel_params.hpp"]


def hipcc_command():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-I" + INCLUDE,
            # packed-FP32 instruction selection is switched off for all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-o", LIB_PATH] + [os.path.join(CSRC, s) for s in SOURCES]


def build(force=True):
    """Compile the library.  With force=False an up-to-date library is kept."""
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.join(INCLUDE, "layoutcopy.h")]
    if not force and os.path.exists(LIB_PATH) and os.path.getmtime(LIB_PATH) >= max(os.path.getmtime(d) for d in deps):
        return LIB_PATH
    subprocess.check_call(hipcc_command(), cwd=CSRC)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
