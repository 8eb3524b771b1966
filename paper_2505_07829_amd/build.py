"""Builds libbb.so (the C-ABI HIP library) in-tree with hipcc for gfx950.

The library has one source per family of kernel instantiations (csrc/*.hip);
they are compiled side by side and linked into one shared object.  Objects go
to `_build/` next to this file (not part of the history)."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbb.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(os.path.dirname(HERE), "include", "bb.h")]


def _obj(src: str) -> str:
    return os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + headers())


def _compile(src: str) -> tuple[str, int, str]:
    res = subprocess.run([HIPCC, *HIPCC_FLAGS, "-c", "-o", _obj(src), src], capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    return src, res.returncode, res.stdout + err


def build(force: bool = True, verbose: bool = False, jobs: int | None = None) -> str:
    """Compile the library.  With force=False only the sources that are newer than their objects
    (a changed header recompiles everything)."""
    if not force and not is_stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    hdr_time = max(os.path.getmtime(h) for h in headers())
    todo = [s for s in sources()
            if force or not os.path.exists(_obj(s)) or os.path.getmtime(_obj(s)) < max(os.path.getmtime(s), hdr_time)]
    jobs = jobs or min(len(todo), os.cpu_count() or 1, 16) or 1
    failed = False
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for src, rc, out in pool.map(_compile, todo):
            if verbose or rc != 0:
                print(f"[{os.path.basename(src)}] rc={rc}\n{out}")
            failed |= rc != 0
    if failed:
        raise RuntimeError("hipcc failed building libbb.so")
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [_obj(s) for s in sources()],
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout + res.stderr)
    if res.returncode != 0:
        raise RuntimeError("linking libbb.so failed")
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--changed" not in sys.argv, verbose=True))
