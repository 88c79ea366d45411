"""Build libdeepgemm_hip.so in-tree with hipcc for gfx950.

Run as ``python -m paper_2304_09049_amd.build`` (or call ``build()``).  The library is placed next
to this file so that it travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdeepgemm_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # only the functions include/deepgemm_hip.h declares are exported
    "-fvisibility=hidden",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the binary32 decisions (Eq. 1: multiply, then add; binary32 tables: add by add) are defined operation by
    # operation: no contraction into fused multiply-adds (hipcc's default is to contract)
    "-ffp-contract=off",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = True, extra_flags=(), jobs: int = 8, incremental: bool = False) -> str:
    """Compile every HIP source (one object each, in parallel) and link one shared library.  Always recompiles,
    unless `incremental` (a development aid): then objects newer than their source and every header are kept."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + list(extra_flags)

    def up_to_date(obj: str) -> bool:
        """The object is newer than every file the compiler read for it (listed in the .d file written beside it)."""
        dep = obj + ".d"
        if not (os.path.exists(obj) and os.path.exists(dep)):
            return False
        with open(dep) as f:
            text = f.read().replace("\\\n", " ")
        files = text.split(":", 1)[1].split() if ":" in text else []
        stamp = os.path.getmtime(obj)
        return bool(files) and all(os.path.exists(x) and os.path.getmtime(x) < stamp for x in files + [os.path.abspath(__file__)])

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        if incremental and up_to_date(obj):
            return obj
        cmd = [hipcc] + flags + ["-MD", "-MF", obj + ".d", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(compile_one, sources()))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    build(extra_flags=[a for a in args if a != "--incremental"], incremental="--incremental" in args)
