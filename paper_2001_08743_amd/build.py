"""Build libcham.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcham.so")
SOURCES = ["cham_api.hip", "lloyd_resident.hip", "lloyd_mfma.hip", "lloyd_stream.hip", "select_snap_synth.hip"]

# -ffp-contract=off: the exact re-evaluation must not fuse multiply and add; fused operations
# in the screening code are written explicitly.  Packed fp32 instructions are switched off.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


# Per-file additions.  The matrix-core kernel takes minima of scores that are finite by construction;
# without the NaN semantics each minimum is one instruction.
FILE_FLAGS = {"lloyd_mfma.hip": ["-fno-honor-nans"]}


def build_lib(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def build_host_sanitized(outdir: str) -> str:
    """A copy of the library whose host code in cham_api.hip (argument checks, planning, staging)
    is built with AddressSanitizer and UndefinedBehaviorSanitizer; device code and the other
    objects are the ordinary ones.  For the CPU-only driver csrc/host_check.c; never loaded by the
    product."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        if src == "cham_api.hip":
            obj = os.path.join(outdir, "cham_api_san.o")
            san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                   "-Xarch_host", "-fno-sanitize-recover=all", "-g"]
            subprocess.run([hipcc, *FLAGS, *san, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
        elif not os.path.exists(obj):
            subprocess.run([hipcc, *FLAGS, *FILE_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj], check=True)
        objs.append(obj)
    lib = os.path.join(outdir, "libcham_san.so")
    # no sanitizer runtime in the shared object: its calls resolve to the runtime of the sanitized driver
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    build_lib(verbose=True, extra=sys.argv[1:])
