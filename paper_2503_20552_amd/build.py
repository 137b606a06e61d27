"""Build libadr.so (the gfx950 HIP library) in-tree with hipcc.

    python -m paper_2503_20552_amd.build [--debug]

Each .hip file under csrc/ is compiled to an object in csrc/_build/ and the
objects are linked into paper_2503_20552_amd/libadr.so.  --debug builds the same
sources with -DADR_DEBUG_BOUNDS into libadr_debug.so (objects in csrc/_build/debug/):
the build that records out-of-range page ids and append positions.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libadr.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed-fp32 instructions are switched off for every device compile.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


DEBUG_LIB = os.path.join(HERE, "libadr_debug.so")


def _compile(name: str, obj_dir: str = OBJ, extra=()) -> str:
    obj = os.path.join(obj_dir, name[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, name), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (name, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, debug: bool = False) -> str:
    obj_dir = os.path.join(OBJ, "debug") if debug else OBJ
    lib = DEBUG_LIB if debug else LIB
    extra = ("-DADR_DEBUG_BOUNDS=1",) if debug else ()
    os.makedirs(obj_dir, exist_ok=True)
    names = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(names))) as ex:
        objs = list(ex.map(lambda n: _compile(n, obj_dir, extra), names))
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, lib)
    if verbose:
        print("built", lib, "from", ", ".join(names))
    return lib


if __name__ == "__main__":
    build(debug="--debug" in sys.argv[1:])
