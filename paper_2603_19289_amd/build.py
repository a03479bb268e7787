"""Builds libmoe_spec.so for gfx950 with hipcc, next to this file."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmoe_spec.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["csrc/moe_spec.cpp", "csrc/route_kernels.hip", "csrc/fused_kernels.hip", "csrc/expert_kernels.hip",
           "csrc/estimator_kernels.hip", "csrc/synth.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


DEMO = os.path.join(HERE, "abi_demo")


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        cmd = [hipcc] + FLAGS + os.environ.get("MOE_SPEC_EXTRA_FLAGS", "").split() + ["-c", os.path.join(HERE, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=HERE)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True, cwd=HERE)
    # the plain C client of the library (C99, host compiler): shows that the header is C and that the
    # boundary needs neither Python nor torch
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    demo = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
            os.path.join(HERE, "csrc/abi_demo.c"), "-o", DEMO, f"-L{HERE}", "-lmoe_spec", f"-L{rocm}/lib",
            "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{rocm}/lib"]
    if verbose:
        print(" ".join(demo), flush=True)
    subprocess.run(demo, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
