"""Build libqg.so (the C-ABI library) from csrc/*.hip for gfx950 with hipcc, in-tree.

Every source is compiled to an object file of its own (in parallel), then linked.  The library
carries an identifier of what it was built from -- a hash over sources, headers and flags,
returned by qg_build_id() -- so that a loader can tell a stale library from a current one
whatever the files' time stamps say.
"""
import glob
import hashlib
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libqg.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt", "-ffp-contract=off",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in registers (used by the GEMV kernels)
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _inputs():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + \
        sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))


def source_id(extra=()) -> str:
    """Hash of everything the library is built from (file names, contents, flags)."""
    h = hashlib.sha256()
    for f in _inputs():
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(f for f in [*FLAGS, *extra] if not f.startswith("-I")).encode())
    return h.hexdigest()[:16]


def is_fresh() -> bool:
    if not os.path.exists(OUT):
        return False
    t = os.path.getmtime(OUT)
    return all(os.path.getmtime(d) <= t for d in _inputs())


def build(force: bool = True, extra=()) -> str:
    if not force and is_fresh():
        return OUT
    os.makedirs(OBJ_DIR, exist_ok=True)
    ident = "-DQG_BUILD_ID=\"%s\"" % source_id(extra)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        subprocess.run([HIPCC, *FLAGS, *extra, ident, "-c", src, "-o", obj], check=True)
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, sources()))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT], check=True)
    return OUT


if __name__ == "__main__":
    print(build())
