"""Builds libsmat.so (host preprocessing + gfx950 kernels + C ABI) in-tree with hipcc."""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libsmat.so")
# registers, scratch and LDS of every kernel as the compiler reported them (written by every build)
RESOURCES = os.path.join(HERE, "_build", "kernel_resources.json")
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


# Kernels that place their own waits for outstanding loads (the tile kernel counts its six loads per step, the
# walks of the per-row kernel theirs): a register spilled inside their loops adds loads the counts do not know
# of and serialises the prefetch (seen once: 79 instead of 53 us).  The build fails if one of them spills.
NO_SPILL = ("spmm_tile_kernel", "spmm_kernel")
_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill|TotalSGPRs|LDS Size \[bytes/block\]): (\S+)")


def _compile(item):
    """Compiles one unit; returns (object file, {kernel: resource usage as the compiler reports it})."""
    name, (src, extra) = item
    obj = os.path.join(OBJ, name + ".o")
    device = src.endswith(".hip")
    cmd = [HIPCC, *FLAGS, *extra, *(["-Rpass-analysis=kernel-resource-usage"] if device else []),
           "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    done = subprocess.run(cmd, check=False, stderr=subprocess.PIPE, text=True)
    usage, kernel, skip = {}, None, 0
    for line in done.stderr.splitlines():
        m = _REMARK.search(line)
        if m:
            if m.group(1) == "Function Name":
                kernel = usage.setdefault(m.group(2), {})
            elif kernel is not None:
                kernel[m.group(1).split(" [")[0]] = int(m.group(2))
            skip = 2                        # the two lines of source context that follow a remark
        elif "-Rpass-analysis=kernel-resource-usage" in line:
            skip = 2
        elif skip > 0 and (line.lstrip().startswith("|") or re.match(r"\s*\d+ \|", line)):
            skip -= 1
        else:
            print(line, file=sys.stderr)
    if done.returncode != 0:
        raise subprocess.CalledProcessError(done.returncode, cmd)
    return obj, usage


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return OUT
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as pool:
        results = list(pool.map(_compile, UNITS.items()))
    objs = [obj for obj, _ in results]
    usage = {}
    for (unit, _), (_, per_kernel) in zip(UNITS.items(), results):
        for kernel, u in per_kernel.items():
            usage[unit + ":" + kernel] = u
    with open(RESOURCES, "w") as f:
        json.dump(usage, f, indent=0, sort_keys=True)
    spilled = [k for k, u in usage.items() if any(n in k for n in NO_SPILL)
               and (u.get("ScratchSize", 0) or u.get("VGPRs Spill", 0))]
    if spilled:
        raise RuntimeError("kernels that must not spill registers do: " + ", ".join(spilled))
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
