"""Builds libpilc.so (hipcc, gfx950 only) next to this file."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libpilc.so")
SOURCES = [os.path.join(CSRC, "pilc.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # no packed-fp32 VALU forms (none are wanted in this integer code anyway)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


DIGEST = LIB + ".digest"   # what the library was built from, so that a stale one is noticed


def source_digest() -> str:
    """SHA-256 over the compile flags and every file the library is built from."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    files = sorted(glob.glob(os.path.join(CSRC, "*")))
    files.append(os.path.join(os.path.dirname(_HERE), "include", "pilc.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def built_digest() -> str:
    """The digest recorded by the build that made the library ('' if none)."""
    try:
        with open(DIGEST) as fh:
            return fh.read().strip()
    except OSError:
        return ""


def build_lib(verbose: bool = False) -> str:
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    digest = source_digest()
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    with open(DIGEST, "w") as fh:
        fh.write(digest + "\n")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
