"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtango.so")
AID_SRC = os.path.join(CSRC, "benchaid", "benchaid.hip")  # measurement aids of the harness: a library of their own
AID_LIB = os.path.join(HERE, "libtango_benchaid.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-ffp-contract=off",  # rounding decisions are specified one fp32 operation at a time
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"),
    "-I" + CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _link(objs, lib):
    tmp = lib + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    os.replace(tmp, lib)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    return obj


def build(verbose: bool = False) -> str:
    """Compile every csrc/*.hip and link libtango.so next to this file; the harness's measurement aids
    (csrc/benchaid/) become libtango_benchaid.so."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
            objs = list(ex.map(_compile, srcs + [AID_SRC]))
        _link(objs[:-1], LIB)
        _link(objs[-1:], AID_LIB)
    except subprocess.CalledProcessError as e:
        sys.stderr.write(e.stderr.decode(errors="replace"))
        raise
    if verbose:
        print("built", LIB)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(AID_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(AID_LIB))
    deps = sources() + [AID_SRC] + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    build(verbose=True)
