"""Compiles the HIP sources under csrc/ for gfx950 into libgids.so (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgids.so")
SOURCES = ["dedup.hip", "cache.hip", "many.hip", "move.hip", "sampler.hip", "api.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the gfx feature flag and says so; that line is noise
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs])
    if verbose:
        print("built", LIB)
    return LIB


def stale() -> bool:
    """True when the library is missing or older than any of its sources."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "gids.h"))
    return any(os.path.getmtime(d) > built for d in deps)


def ensure_built() -> str:
    """Build when no library is there yet or a source is newer than it (tests, the smoke check and the
    benchmark call this).  A machine without hipcc uses the library it was given."""
    if stale():
        import shutil
        if shutil.which("hipcc") is None:
            if os.path.exists(LIB):
                return LIB
            raise RuntimeError("libgids.so is missing and hipcc is not on PATH")
        return build()
    return LIB


if __name__ == "__main__":
    build(verbose=True)
