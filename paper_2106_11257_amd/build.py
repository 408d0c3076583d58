"""Builds libbtard.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree.

The sources are compiled to objects side by side (one translation unit per family of kernel
instantiations) and linked into one shared library."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbtard.so")
SOURCES = ["btard_api.hip", "tables_pass.hip", "tables_finish.hip", "tables_fused.hip",
           "tables_verify.hip", "tables_median.hip"]
HEADERS = ["kernels_common.h", "cc_kernels.h", "verify_kernels.h", "fused_kernels.h",
           "gram_kernels.h", "median_kernels.h", "hash_kernels.h", "dispatch.h",
           os.path.join("..", "..", "include", "btard.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(p) > t for p in deps)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    return res.stdout


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library.  Returns its path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("BTARD_EXTRA_HIPCC_FLAGS", "").split()
    os.makedirs(OBJ, exist_ok=True)
    objects = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    jobs = int(os.environ.get("MAX_JOBS", "0")) or min(len(SOURCES), os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + extra +
                                      ["-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                      zip(SOURCES, objects)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objects, verbose)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
