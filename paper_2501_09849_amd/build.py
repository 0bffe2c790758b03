"""Builds libcdl.so (the HIP kernels and the C boundary) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libcdl.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions stay off: the compiler must not form v_pk_*_f32 from float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fusing of a*b+c: the kernels spell out every fused multiply-add they rely on
    # (the error-free splits in the quantizer need the plain product and the plain difference)
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


HASH_PATH = LIB_PATH + ".srchash"


def _deps():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + sorted(glob.glob(os.path.join(_ROOT, "include", "*.h")))


def source_hash() -> str:
    """sha256 over the compiler flags and every source and header the library is built from (contents, not
    time stamps: a copy of the tree to another machine keeps it)."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for path in _deps():
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when libcdl.so is missing or was not built from the sources now in the tree."""
    if not (os.path.exists(LIB_PATH) and os.path.exists(HASH_PATH)):
        return True
    with open(HASH_PATH) as f:
        return f.read().strip() != source_hash()


def build_lib(verbose: bool = False) -> str:
    """Compile every .hip source into libcdl.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"), "-I", CSRC] + sources() + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and res.stdout.strip():
        print(res.stdout)
    os.replace(tmp, LIB_PATH)
    if LIB_PATH.endswith(os.path.join(os.path.basename(_HERE), "libcdl.so")):
        with open(HASH_PATH, "w") as f:
            f.write(source_hash() + "\n")
    return LIB_PATH


if __name__ == "__main__":
    print(build_lib(verbose=True))
