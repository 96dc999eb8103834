"""Builds the HIP library for gfx950 in-tree: ``python -m paper_2210_02574_amd.build``."""
from __future__ import annotations

import concurrent.futures
import glob
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhe_gfx950.so")
# one object per ring size and kernel family: they compile in parallel
SOURCES = (
    # (source, extra defines, object name), the slowest first
    [("dev_cols.hip", ["-DHE_LOGN=%d" % n, "-DHE_PRO=%d" % p], "dev_cols%d_%d" % (n, p)) for n in (17, 16) for p in (4, 2, 1, 5, 3, 0)]
    # the corrected base conversions: kernels of their own
    + [("dev_cols.hip", ["-DHE_LOGN=%d" % n, "-DHE_PRO=%d" % p, "-DHE_EX=1"], "dev_cols_ex%d_%d" % (n, p)) for n in (17, 16) for p in (4, 2, 1)]
    + [(s, [], os.path.splitext(s)[0]) for s in ("dev_n12.hip", "dev_n16_blocks.hip", "dev_n17_blocks.hip", "device.hip", "host.cpp")]
)
OBJDIR = os.path.join(HERE, "_build")
STAMP = LIB + ".srchash"  # hash of the sources the built library was compiled from


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


CODEGEN_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off",
]


def _flags():
    # HE_EXTRA_HIPCC_FLAGS: diagnostics such as -Rpass-analysis=kernel-resource-usage (not part of the source hash)
    return CODEGEN_FLAGS + [
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    ] + os.environ.get("HE_EXTRA_HIPCC_FLAGS", "").split()


def _inputs():
    """Every file the library is built from."""
    return sorted(glob.glob(os.path.join(CSRC, "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))


def source_hash() -> str:
    h = hashlib.sha256()
    for f in _inputs():
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(CODEGEN_FLAGS).encode())
    return h.hexdigest()


def build(verbose: bool = False, jobs: int | None = None, only=None) -> str:
    """Compile every source for gfx950 and link the shared library (always recompiles).  `only`: object names
    to recompile while the other objects of the last build are reused (a development shortcut)."""
    os.makedirs(OBJDIR, exist_ok=True)
    stamp = source_hash()
    jobs = jobs or min(len(SOURCES), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1)))

    def compile_one(item) -> str:
        src, defines, name = item
        obj = os.path.join(OBJDIR, name + ".o")
        if only is not None and name not in only and os.path.exists(obj):
            return obj
        cmd = [hipcc()] + _flags() + defines + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB + ".tmp", "-lpthread"]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    os.replace(LIB + ".tmp", LIB)
    with open(STAMP, "w") as fh:
        fh.write(stamp + "\n")
    return LIB


def is_stale() -> bool:
    """True when no library is built or its sources have changed since (by content, not by time stamp)."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as fh:
        return fh.read().strip() != source_hash()


def ensure_built() -> str:
    """Loads what is built; compiles only when nothing is.  A library built from other sources than the present ones is an error
    rather than a silent run of stale kernels (rebuild with ``python -m paper_2210_02574_amd.build``)."""
    if not os.path.exists(LIB):
        return build()
    if is_stale() and not os.environ.get("HE_ALLOW_STALE_LIB"):
        raise RuntimeError(
            f"{LIB} was built from other sources: rebuild with `python -m paper_2210_02574_amd.build` "
            "(or set HE_ALLOW_STALE_LIB=1 to load it anyway)"
        )
    return LIB


if __name__ == "__main__":
    names = [a for a in sys.argv[1:] if not a.startswith("-")]
    print(build(verbose="-v" in sys.argv, only=names or None))
