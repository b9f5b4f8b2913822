"""Builds libstx.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libstx.so")
CSRC = os.path.join(HERE, "csrc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         # keep hipcc from forming packed-fp32 instructions on its own
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip"))) + sorted(glob.glob(os.path.join(CSRC, "*.cpp")))


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build_lib(verbose: bool = False) -> str:
    """Every source is compiled (one hipcc per file, side by side) and the objects are linked into libstx.so."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    jobs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        jobs.append((["hipcc", *compile_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        outs = list(pool.map(lambda j: _run(j[0]), jobs))
    outs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *(o for _, o in jobs), "-o", LIB]))
    out = "\n".join(o for o in outs if o.strip())
    if verbose and out:
        print(out)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
