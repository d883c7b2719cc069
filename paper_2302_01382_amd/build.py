"""Builds libmpq.so from csrc/*.hip with hipcc for gfx950 (in-tree, next to this file).

Every source is compiled to an object of its own (side by side, one hipcc per source) and the
objects are linked into the shared library.  `build_lib()` recompiles everything; with
`incremental=True` only the sources that changed since their object was written are recompiled
(a development convenience, never used by the driver's build check).
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
# MPQ_SANITIZE_HOST=1: a second copy of the library whose HOST code (argument checks, plan
# builders, searches, host arithmetic) is instrumented with the address and undefined-behaviour
# sanitizers; device code is unchanged.  For the CPU test suite on a GPU-less machine:
#   LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" \
#       ASAN_OPTIONS=detect_leaks=0 MPQ_SANITIZE_HOST=1 python -m pytest tests -m "not gpu"
SANITIZE_HOST = os.environ.get("MPQ_SANITIZE_HOST", "0") not in ("", "0")
OBJ = os.path.join(HERE, "_build_san" if SANITIZE_HOST else "_build")
LIB = os.path.join(HERE, "libmpq_san.so" if SANITIZE_HOST else "libmpq.so")
# (the function-type and vptr checks are left out: the runtime that is preloaded is gcc's, which
# has no handler for them)
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize=function,vptr", "-Xarch_host", "-fno-omit-frame-pointer"]

# -ffp-contract=off: every fused multiply-add in the kernels is written explicitly.
# packed fp32 instructions are switched off for the device compiler (the host pass warns that it
# does not know the feature; harmless).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def find_hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libmpq cannot be built on this machine")
    return exe


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers():
    return glob.glob(os.path.join(CSRC, "*.hpp")) + [os.path.join(ROOT, "include", "mpq.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + headers())


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_lib(verbose: bool = False, incremental: bool = False, jobs: int = 8) -> str:
    """Compiles the sources (all of them unless `incremental`), links libmpq.so, returns its path."""
    hipcc = find_hipcc()
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in headers())
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            todo.append([hipcc, *HIPCC_FLAGS, *(SAN_FLAGS if SANITIZE_HOST else []), "-I", os.path.join(ROOT, "include"),
                         "-I", CSRC, "-c", src, "-o", obj])
    # stale objects of sources that no longer exist must not be linked
    for stray in set(glob.glob(os.path.join(OBJ, "*.o"))) - set(objs):
        os.remove(stray)
    with ThreadPoolExecutor(max(1, jobs)) as ex:
        list(ex.map(lambda c: _run(c, verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *(SAN_FLAGS if SANITIZE_HOST else []), "-o", LIB + ".tmp",
          *objs], verbose)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True, incremental="--incremental" in sys.argv))
    sys.exit(0)
