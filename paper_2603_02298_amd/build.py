"""Builds liblayoutcopy.so (host algebra + planners + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_PATH = os.path.join(HERE, "liblayoutcopy.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["layout.cpp", "algebra.cpp", "semimodule.cpp", "plan.cpp", "replay.cpp", "gemm_plan.cpp", "gemm_replay.cpp", "capi.cpp",
           "gemm_capi.cpp", "kernels.hip", "gemm_kernels.hip", "gemm_inst_bf16_256.hip", "gemm_inst_bf16_128.hip",
           "gemm_inst_f16_256.hip", "gemm_inst_f16_128.hip"]
HEADERS = ["layout.hpp", "algebra.hpp", "semimodule.hpp", "plan.hpp", "kernel_params.hpp", "gemm_plan.hpp", "gemm_params.hpp", "plan_cache.hpp"]
KERNEL_HEADERS = {"gemm_kernel.hpp": "gemm_inst_"}   # header -> prefix of the only sources that include it


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


# kernels.hip: the leading scalar kernel arguments (up to 14 dwords) are preloaded into scalar registers at wavefront
# start where the firmware supports it; the compiler keeps a prologue that loads them for firmware that does not
EXTRA_FLAGS = {"kernels.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=14"]}


def compile_command(source):
    return [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE,
            # packed-FP32 instruction selection is switched off for all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + EXTRA_FLAGS.get(source, []) + [
            "-c", os.path.join(CSRC, source), "-o", os.path.join(OBJ_DIR, source + ".o")]


def link_command():
    return [_hipcc(), "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB_PATH] + [os.path.join(OBJ_DIR, s + ".o") for s in SOURCES]


def build(force=True):
    """Compile the library: one object per source (in parallel), then link.  With force=False objects and
    library that are newer than every source and header are kept."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    common = [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(INCLUDE, "layoutcopy.h")]
    newest_common = max(os.path.getmtime(d) for d in common)
    todo = []
    for s in SOURCES:
        obj = os.path.join(OBJ_DIR, s + ".o")
        src_time = max(newest_common, os.path.getmtime(os.path.join(CSRC, s)))
        for header, prefix in KERNEL_HEADERS.items():
            if s.startswith(prefix):
                src_time = max(src_time, os.path.getmtime(os.path.join(CSRC, header)))
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < src_time:
            todo.append(s)
    if todo:
        with ThreadPoolExecutor(max_workers=min(8, len(todo))) as pool:
            list(pool.map(lambda s: subprocess.check_call(compile_command(s), cwd=CSRC), todo))
    if todo or not os.path.exists(LIB_PATH):
        subprocess.check_call(link_command(), cwd=CSRC)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
