"""Builds libhbcsf.so (host format builder + gfx950 kernels + C ABI) in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
SO = os.path.join(HERE, "libhbcsf.so")

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False) -> str:
    """Compiles every source each time it is called and links the shared library."""
    objs = []
    inc = ["-I", INCLUDE, "-I", CSRC]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    o = os.path.join(CSRC, "hbcsf_format.o")
    run(["g++", "-O3", "-std=c++17", "-fPIC", "-fopenmp", "-c", os.path.join(CSRC, "hbcsf_format.cpp"), "-o", o] + inc)
    objs.append(o)
    # the kernels are compiled once per (lanes per row, order) pair, in parallel
    jobs = []
    for g in (2, 4, 8, 16, 32):
        for n in (3, 4, 5):
            o = os.path.join(CSRC, f"hbcsf_kernels_g{g}_n{n}.o")
            defs = [f"-DHBCSF_G={g}", f"-DHBCSF_N={n}"] + (["-DHBCSF_WITH_DEFINE"] if (g, n) == (8, 3) else [])
            jobs.append(["hipcc"] + HIP_FLAGS + inc + defs + ["-c", os.path.join(CSRC, "hbcsf_kernels.hip"), "-o", o])
            objs.append(o)
    # fp64 factor matrices and output: ranks 16, 32, 64 = 8, 16, 32 lanes of 16 bytes per row
    for g in (8, 16, 32):
        for n in (3, 4, 5):
            o = os.path.join(CSRC, f"hbcsf_kernels_f64_g{g}_n{n}.o")
            defs = [f"-DHBCSF_G={g}", f"-DHBCSF_N={n}", "-DHBCSF_F64"]
            jobs.append(["hipcc"] + HIP_FLAGS + inc + defs + ["-c", os.path.join(CSRC, "hbcsf_kernels.hip"), "-o", o])
            objs.append(o)
    for name in ("hbcsf_capi", "hbcsf_als", "hbcsf_devbuild"):
        o = os.path.join(CSRC, name + ".o")
        jobs.append(["hipcc"] + HIP_FLAGS + inc + ["-c", os.path.join(CSRC, name + ".hip"), "-o", o])
        objs.append(o)
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4))))
    with ThreadPoolExecutor(workers) as pool:
        list(pool.map(run, jobs))
    run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", SO] + objs + ["-lgomp"])
    return SO


if __name__ == "__main__":
    print(build(verbose=True))
