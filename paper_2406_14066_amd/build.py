"""Builds the HIP library (``libspec_verify.so``) in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspec_verify.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fgpu-flush-denormals-to-zero",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# step_kernel.hip holds dozens of kernel variants; it is compiled once per part (see SPEC_STEP_PART
# in that file), in parallel with the other sources, and the objects are linked.
STEP_KERNEL = "step_kernel.hip"
STEP_PARTS = 5


def compile_jobs(objdir: str):
    """(command, object file) for every translation unit of the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    base = [hipcc] + flags + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c"]
    jobs = []
    for src in sources():
        stem = os.path.splitext(os.path.basename(src))[0]
        if os.path.basename(src) == STEP_KERNEL:
            for part in range(STEP_PARTS):
                obj = os.path.join(objdir, "%s_part%d.o" % (stem, part))
                jobs.append((base + ["-DSPEC_STEP_PART=%d" % part, "-o", obj, src], obj))
        else:
            obj = os.path.join(objdir, stem + ".o")
            jobs.append((base + ["-o", obj, src], obj))
    return jobs


def build_library(verbose: bool = False) -> str:
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = tempfile.mkdtemp(prefix="spec_verify_build_")
    try:
        jobs = compile_jobs(objdir)

        def run(job):
            if verbose:
                print(" ".join(job[0]))
            subprocess.run(job[0], check=True)
            return job[1]

        with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 4, 16)) as pool:
            objects = list(pool.map(run, jobs))
        tmp = LIB + ".tmp.%d" % os.getpid()
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objects
        if verbose:
            print(" ".join(link))
        subprocess.run(link, check=True)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
