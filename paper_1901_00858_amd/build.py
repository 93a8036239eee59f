"""Compile libhgc.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libhgc.so")
SOURCES = ["api.hip", "igemm_tables.hip", *["igemm_%s_%d.hip" % (k, i) for k in ("raw", "packed") for i in range(4)], "direct.hip", "pack.hip", "inner_product.hip", "smallc.hip",
           "batch_norm.hip", "max_pool.hip", "pointwise.hip"]
HEADERS = [os.path.join(CSRC, "hgc_internal.h"), os.path.join(CSRC, "igemm_kernel.h"), os.path.join(CSRC, "tile_store.h"),
           os.path.join(ROOT, "include", "hgc.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-value",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True, verbose: bool = False, incremental: bool = False) -> str:
    """Compile every HIP source into paper_1901_00858_amd/libhgc.so. Returns its path.

    incremental: keep the object files (under _build/) and recompile only the sources that are newer
    than theirs, or whose headers are; for work on one kernel.  The default compiles everything.
    """
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build") if incremental else CSRC
    os.makedirs(objdir, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(objdir, s.replace(".hip", ".o"))
        objs.append(obj)
        src = os.path.join(CSRC, s)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out, file=sys.stderr)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    if not incremental:
        for o in objs:
            os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True, incremental="--incremental" in sys.argv[1:]))
