"""Builds libgroot.so (host C++ + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libgroot.so")
SOURCES = [os.path.join(CSRC, "groot_host.cpp"), os.path.join(CSRC, "groot_kernels.hip"),
           os.path.join(CSRC, "groot_sage.hip"), os.path.join(CSRC, "groot_plan_device.hip"),
           os.path.join(CSRC, "groot_ld_pipe.hip"), os.path.join(CSRC, "groot_regrow_device.hip"),
           os.path.join(CSRC, "groot_sage_pipe.hip"), os.path.join(CSRC, "groot_compress.hip"),
           os.path.join(CSRC, "groot_hd_sched_device.hip"), os.path.join(CSRC, "groot_sage_wgrad.hip")]
HEADERS = [os.path.join(CSRC, "groot_internal.h"), os.path.join(CSRC, "groot_device.h"),
           os.path.join(ROOT, "include", "groot.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > built for p in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Compiles every source to an object of its own (in parallel, at most 8 at a time) under a build folder in the
    temporary directory, then links the shared library in-tree."""
    import concurrent.futures
    import tempfile

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [
        "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
        # packed fp32 instructions are kept out of the generated code
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    ]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout)
        if verbose and lines:
            print("\n".join(lines))

    with tempfile.TemporaryDirectory(prefix="groot_build_") as tmp:
        objects = [os.path.join(tmp, os.path.splitext(os.path.basename(src))[0] + ".o") for src in SOURCES]
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
            jobs = [pool.submit(run, [hipcc] + flags + ["-c", src, "-o", obj]) for src, obj in zip(SOURCES, objects)]
            for job in jobs:
                job.result()
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objects + ["-lpthread"])
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
