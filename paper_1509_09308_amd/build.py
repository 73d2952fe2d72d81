"""Compiles the HIP sources under csrc/ into libwino.so for gfx950 (in-tree, next to this file)."""
import glob
import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwino.so")
HASH_PATH = LIB_PATH + ".srchash"     # written next to the library by build()
CSRC = os.path.join(_HERE, "csrc")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose=False):
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = list(HIPCC_FLAGS)
    cmd = [hipcc] + flags + ["-o", LIB_PATH] + sources()
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    with open(HASH_PATH, "w") as fh:
        fh.write(source_hash() + "\n")
    return LIB_PATH


def inputs():
    """Every file the library is compiled from."""
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + \
        [os.path.join(os.path.dirname(_HERE), "include", "wino.h")]


def source_hash():
    """Hash of the contents of inputs() and of the compiler flags (file times do not survive every copy)."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for f in inputs():
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def built_hash():
    """source_hash() of the sources the present library was compiled from, or None."""
    try:
        with open(HASH_PATH) as fh:
            return fh.read().strip()
    except OSError:
        return None


def stale():
    """True when the library is missing or was compiled from other sources than the present ones."""
    return not os.path.exists(LIB_PATH) or built_hash() != source_hash()


def ensure_built():
    """Builds when the library is missing or does not match the sources; returns its path."""
    if stale():
        build()
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
