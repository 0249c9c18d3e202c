"""Build the HIP library (libdd.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libdd.so")
SOURCES = ["dd_api.hip", "verify.hip", "attention_mfma.hip", "attention_wide.hip", "attention_stream.hip", "attention_f32.hip", "cache.hip"]
HEADERS = ["dd_internal.h", "attention_common.h", os.path.join("..", "..", "include", "dd.h")]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         # packed-fp32 instructions are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(p) > t for p in deps)


def build_library(force: bool = True, verbose: bool = False, extra_flags=()) -> str:
    """Compile every kernel source into one shared library.  Returns its path."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra_flags) + ["-o", LIB] + [os.path.join(CSRC, f) for f in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True, extra_flags=sys.argv[1:]))
