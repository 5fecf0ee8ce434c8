"""Builds paper_2510_27656_amd/csrc/libflmoe.so with hipcc for gfx950 (in-tree)."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libflmoe.so")
SOURCES = ["flmoe.hip"]
HEADERS = ["common.h", "kernels_layout.h", "kernels_shuffle.h", "../../include/flmoe.h"]


def lib_path() -> str:
    return LIB


def source_hash() -> str:
    """Identifies the sources the library is built from.  The build passes it to the
    compiler, the library returns it from fl_moe_build_id(), so a loaded binary can be
    checked against the tree (and a stored profile against the binary that is timed)."""
    h = hashlib.sha256()
    for f in sorted(SOURCES + HEADERS):
        h.update(f.encode())
        h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()[:16]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Always compiles (cross-compiles without a GPU)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function", f'-DFLMOE_BUILD_ID="{source_hash()}"',
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
