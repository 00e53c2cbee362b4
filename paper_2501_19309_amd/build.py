"""Compile the HIP sources into libjdverify.so (in-tree, gfx950 only).

    python -m paper_2501_19309_amd.build
"""

from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libjdverify.so")

SOURCES = ["jd_verify_api.hip", "lmhead_skinny.hip", "lmhead_gemm.hip", "lmhead_gemm_dma.hip", "verify_tail.hip", "device_probes.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


CABI_CHECK_SRC = os.path.join(os.path.dirname(HERE), "tests", "cabi_check.cpp")
CABI_CHECK_PATH = os.path.join(HERE, "jd_cabi_check")


def build_cabi_check(verbose: bool = False) -> str:
    """The stand-alone C++ caller of the C ABI that the GPU tests run (tests/cabi_check.cpp): host code only,
    linked against libjdverify.so next to it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", CABI_CHECK_SRC, "-L" + HERE, "-ljdverify",
           "-Wl,-rpath,$ORIGIN", "-o", CABI_CHECK_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building jd_cabi_check")
    return CABI_CHECK_PATH


def build_library(verbose: bool = False) -> str:
    """One hipcc process per source file, side by side (no device code is shared between the files except through
    headers, so no relocatable device code is needed), then one link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    tmp = tempfile.mkdtemp(prefix="jdverify_build_")
    try:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc] + HIPCC_FLAGS + ["-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                sys.stderr.write(res.stdout + res.stderr)
                raise RuntimeError("hipcc failed compiling " + os.path.basename(src))
            if verbose and res.stderr.strip():
                print(res.stderr)
            return obj

        jobs = max(1, min(len(srcs), int(os.environ.get("MAX_JOBS", "0")) or (os.cpu_count() or 2)))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, srcs))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError("hipcc failed linking libjdverify.so")
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_cabi_check(verbose=True))
