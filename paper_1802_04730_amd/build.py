"""Build libtc355.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtc355.so")
STAMP = LIB + ".srchash"  # hash of the sources the library was built from

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps():
    return sorted(glob.glob(os.path.join(CSRC, "*.h*"))) + [os.path.join(HERE, "..", "include", "tc355.h")]


def source_hash() -> str:
    """Hash of everything the library is compiled from (file contents, not time stamps: a copy of the tree keeps it)."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for d in _deps():
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True if there is no built library or it was built from other sources than the tree holds now."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_hash()


def hipcc_path() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def have_hipcc() -> bool:
    return os.access(hipcc_path(), os.X_OK)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into libtc355.so; returns the library path."""
    if not force and not is_stale():
        return LIB
    hipcc = hipcc_path()
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout + r.stderr)
    with open(STAMP, "w") as f:
        f.write(source_hash() + "\n")
    if verbose:
        noise = "is not a recognized feature for this target"
        for line in r.stderr.splitlines():
            if noise not in line:
                print(line)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
