"""Builds libactq.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libactq.so")
SOURCES = ["actq_api.cpp", "actq_kernels.hip", "actq_context.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # the scaling step of the quantizer is a separately rounded subtract and multiply
    "-ffp-contract=off",
    # inputs are finite by contract: lets min/max compile to single v_min/v_max (and fold
    # into DPP forms) instead of quieting signalling NaNs first
    "-fno-honor-nans",
    # keep binary32 arithmetic on the scalar-issue VALU forms
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # "#pragma unroll" on loops whose trip count is a template parameter that may be a run-time value
    "-Wno-pass-failed",
]


def source_hash() -> str:
    """Digest of everything the binary depends on: the sources, the public and internal headers
    and the compiler flags."""
    import hashlib
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".cpp", ".h"))]
    files.append(os.path.join(ROOT, "include", "actq.h"))
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()[:16]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libactq cannot be built")
    return exe


def build(verbose: bool = False) -> str:
    """Compile every source of the library; always recompiles."""
    tmp = LIB + f".{os.getpid()}.tmp"
    cmd = [hipcc(), *HIPCC_FLAGS, f'-DACTQ_SOURCE_HASH="{source_hash()}"',
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
