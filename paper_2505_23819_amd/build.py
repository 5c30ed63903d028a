"""Build the HIP library in-tree: hipcc cross-compiles for gfx950 without a GPU."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libll355.so")
SOURCES = ["f2.cpp", "plan.cpp", "plan_vec.cpp", "plan_pull.cpp", "plan_tr.cpp", "algebra.cpp", "families.cpp", "options.cpp", "run.cpp", "capi.cpp", "kernels.hip"]
HEADERS = ["f2.hpp", "layout.hpp", "plan.hpp", "kernels.hpp", os.path.join("..", "..", "include", "ll.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    "-Wno-unused-parameter",
    # packed FP32 instructions are never wanted here (pure data movement)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP/C++ source into libll355.so (always recompiles when force=True)."""
    if not force and not is_stale():
        return LIB
    cmd = [HIPCC] + FLAGS + [os.path.join(CSRC, f) for f in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
