"""Build step of the HIP library: hipcc cross-compiles for gfx950 (no GPU needed).

Every source is compiled to an object of its own (in parallel) and the objects are linked into
``libdfss.so`` next to this file.  ``build()`` compiles everything; ``build(incremental=True)``
recompiles only the sources that are newer than their object (a header change recompiles all).
"""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdfss.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # inputs are finite by contract: without these every fmaxf/fminf is wrapped in two extra
    # canonicalising v_max_f32 (signalling-NaN quieting of IEEE mode)
    "-fno-honor-nans", "-mno-amdgpu-ieee",
    # the asynchronous-copy helper sets M0 inside its inline assembly and says so in the clobber list;
    # the compiler notes on every instantiation that M0 is a reserved register
    "-Wno-inline-asm",
    "-I" + os.path.join(ROOT, "include"),
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers():
    return (sorted(glob.glob(os.path.join(CSRC, "*.hpp"))) + sorted(glob.glob(os.path.join(CSRC, "*.h")))
            + [os.path.join(ROOT, "include", "dfss.h")])


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _show(cmd, res):
    print(" ".join(cmd))
    print(res.stdout)
    print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))


def _compile(src: str, obj: str, verbose: bool):
    cmd = [_hipcc(), *HIPCC_FLAGS, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        _show(cmd, res)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed compiling {os.path.basename(src)}")


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every kernel source and link libdfss.so next to this file."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in headers())
    jobs, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            jobs.append((src, obj))
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for f in [pool.submit(_compile, s, o, verbose) for s, o in jobs]:
            f.result()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        _show(cmd, res)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libdfss.so")
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + headers())


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
