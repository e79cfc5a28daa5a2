"""Compile libbsp.so (host packer + HIP kernels) for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libbsp.so")


def sources():
    c = os.path.join(PKG, "csrc")
    return sorted(glob.glob(os.path.join(c, "*.cpp")) + glob.glob(os.path.join(c, "*.hip")))


def build(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Always recompiles; returns the path of the shared library."""
    LIB = out
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
           # packed fp32 arithmetic is kept out of all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
           "-o", LIB + ".tmp"] + list(extra_flags) + sources()
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("-o", "--out", default=LIB)
    ap.add_argument("flags", nargs="*", help="extra hipcc flags, e.g. -DNAME")
    a, unknown = ap.parse_known_args()
    print(build(verbose=True, extra_flags=a.flags + unknown, out=os.path.abspath(a.out)))
