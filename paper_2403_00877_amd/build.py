"""Build libdmt.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdmt.so")

FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
OBJDIR = os.path.join(HERE, "_build")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, jobs: int = None) -> str:
    """Compile every source to an object (in parallel), then link libdmt.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJDIR, os.path.basename(s)[:-4] + ".%d.o" % os.getpid()) for s in srcs]

    def compile_one(pair):
        src, obj = pair
        cmd = [hipcc] + FLAGS + ["-c", "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    jobs = jobs or min(len(srcs), max(1, min(16, os.cpu_count() or 1)))
    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(compile_one, zip(srcs, objs)))
        tmp = LIB + ".tmp%d" % os.getpid()
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, LIB)
        with open(STAMP, "w") as f:
            f.write(source_digest() + "\n")
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return LIB


def source_digest() -> str:
    """SHA-256 over everything the library is built from (sources, headers, flags)."""
    import hashlib
    h = hashlib.sha256()
    deps = sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(ROOT, "include", "dmt.h")]
    for d in deps:
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    h.update(" ".join(FLAGS[:-4]).encode())          # (not the include paths, which name this checkout)
    return h.hexdigest()


STAMP = LIB + ".stamp"


def is_stale() -> bool:
    """True when libdmt.so is missing or was not built from the sources in the tree (by content,
    not by file time: a copied tree keeps no trustworthy times)."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_digest()


if __name__ == "__main__":
    print(build(verbose=True))
