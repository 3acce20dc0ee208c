"""Builds libcusa.so (gfx950) in-tree from csrc/ with hipcc."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libcusa.so")
SOURCES = [os.path.join(CSRC, "cusa.hip")]
HEADERS = [os.path.join(CSRC, "cusa_kernels.hpp"),
           os.path.join(os.path.dirname(_HERE), "include", "cusa.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the leading kernel arguments arrive in SGPRs with the wave instead of through a first load
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libcusa cannot be built")
    return exe


def source_id() -> str:
    """Digest of everything the library is compiled from (sources, headers, flags); the library
    carries the digest it was built from (cusa_build_id), which is how a stale binary is told."""
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()[:16]


def build_lib(force: bool = True, extra_flags=()) -> str:
    """Compile the library; with force=False only when it is missing."""
    if not force and os.path.exists(LIB):
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc(), *HIPCC_FLAGS, f'-DCUSA_BUILD_ID="{source_id()}"', *extra_flags, "-o", tmp, *SOURCES]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(True))
