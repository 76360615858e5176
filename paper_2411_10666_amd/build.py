"""Compile the HIP library for gfx950 in-tree (``paper_2411_10666_amd/libsam_hip.so``)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsam_hip.so")
SOURCES = ["sam_api.hip", "sam_kernels.hip", "sam_tree.hip", "sam_membench.hip", "sam_host.cpp"]
HEADERS = ["sam_layout.h", "sam_device.h", "sam_host.h", "sam_membench.h", os.path.join("..", "..", "include", "sam.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def source_digest() -> str:
    """Digest of every source and header the library is compiled from.  It is compiled
    into the library (sam_build_id) so that a loaded binary can be told from one that
    is older than the sources beside it, whatever the file times say."""
    import hashlib
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(f.encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def build(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    build_id = '-DSAM_BUILD_ID="%s"' % source_digest()
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + HIPCC_FLAGS + [build_id, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
