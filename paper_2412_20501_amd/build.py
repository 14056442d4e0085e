"""Builds libtokenring.so (HIP, gfx950 only) in-tree with hipcc.

The library carries a hash of everything it was compiled from (kernel sources, internal and
public headers, compiler flags): tr_version() reports it, and ensure_built() recompiles when
the hash found inside an existing library differs from the hash of the sources on disk, so a
test or benchmark run can never silently exercise a stale binary.
"""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(PKG_DIR, "libtokenring.so")
SOURCES = ["api.hip", "block_attn.hip", "merge.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
_HASH_TAG = b"TR_SOURCE_HASH="


def source_hash() -> str:
    """Hex digest (16 characters) over every file of csrc/ and include/ plus the compiler flags."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for folder in (CSRC, INCLUDE):
        for name in sorted(os.listdir(folder)):
            path = os.path.join(folder, name)
            if os.path.isfile(path) and name.endswith((".hip", ".h", ".hpp", ".inc")):
                h.update(name.encode() + b"\0")
                with open(path, "rb") as f:
                    h.update(f.read())
                h.update(b"\0")
    return h.hexdigest()[:16]


def library_hash(path: str = LIB_PATH):
    """The source hash embedded in a built library (read from the file, nothing is loaded); None if absent."""
    if not os.path.exists(path):
        return None
    with open(path, "rb") as f:
        m = re.search(re.escape(_HASH_TAG) + rb"([0-9a-f]{16})", f.read())
    return m.group(1).decode() if m else None


def build_library(verbose: bool = False) -> str:
    """Compile every kernel source into one shared library; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, f'-DTR_SOURCE_HASH_STR="{source_hash()}"', "-I", INCLUDE, "-I", CSRC,
           "-o", tmp, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, LIB_PATH)      # atomic: a concurrent reader never sees a half-written library
    return LIB_PATH


def ensure_built() -> str:
    """Build unless a library compiled from exactly the sources on disk is already there."""
    if library_hash() == source_hash():
        return LIB_PATH
    return build_library()


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
