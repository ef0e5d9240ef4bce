"""Builds libsmat.so (host preprocessing + gfx950 kernels + C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libsmat.so")
# a plain-C program that uses the library through include/smat.h alone (no Python in the process)
EXAMPLE_SRC = os.path.join(HERE, "..", "examples", "c_abi_example.c")
EXAMPLE_OUT = os.path.join(HERE, "c_abi_example")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
# The per-row kernel starts with a chain of dependent loads (launch record -> slot table -> rows
# of B); having the dispatcher place its leading arguments in scalar registers takes the load of
# the arguments themselves off the front of that chain.
PRELOAD = ["-mllvm", "-amdgpu-kernarg-preload-count=16"]
# object name -> (source, extra flags)
UNITS = {
    "api": ("api.cpp", []),
    "preprocess": ("preprocess.cpp", []),
    "kernels": ("kernels.hip", PRELOAD),
    "kernels_narrow": ("kernels_narrow.hip", PRELOAD),
    # the per-row kernel for the 8-bit operand types: one object per type, built side by side
    "kernels_e4m3": ("kernels_8bit.hip", ["-DSMAT_8BIT_DT=2", *PRELOAD]),
    "kernels_e5m2": ("kernels_8bit.hip", ["-DSMAT_8BIT_DT=3", *PRELOAD]),
    "kernels_i8": ("kernels_8bit.hip", ["-DSMAT_8BIT_DT=4", *PRELOAD]),
    # the dense kernel keeps 128 accumulator registers per lane next to ~90 others: have the
    # MFMA results live in ordinary VGPRs instead of being shuffled between the two register files
    "kernels_dense": ("kernels_dense.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form=1", *PRELOAD]),
    # the tile-step probe is the tile kernel's loop: same flag
    "probes": ("probes.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]),
    "ablation": ("ablation.hip", []),
}
HEADERS = ["kernels.h", "preprocess.h", "pack_layout.h", "spmm_rows.h", os.path.join("..", "..", "include", "smat.h"),
           os.path.join("..", "..", "include", "smat_bench.h"), "mfma_types.h"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(OUT):
        return True
    built = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, f) for f in sorted({src for src, _ in UNITS.values()}) + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > built for d in deps)


def _compile(item):
    name, (src, extra) = item
    obj = os.path.join(OBJ, name + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.run(cmd, check=True)
    return obj


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return OUT
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(_compile, UNITS.items()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    if os.path.exists(EXAMPLE_SRC):
        cmd = [os.environ.get("CC", "gcc"), "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", EXAMPLE_SRC,
               "-I" + os.path.join(HERE, "..", "include"), "-I" + os.path.join(ROCM, "include"),
               "-L" + HERE, "-lsmat", "-L" + os.path.join(ROCM, "lib"), "-lamdhip64",
               "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-o", EXAMPLE_OUT]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
