"""Builds libmmvseg.so (HIP, gfx950 only) next to this file with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "mmvseg.hip")
LIB = os.path.join(HERE, "libmmvseg.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"),
]


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compiles the library; `extra` adds compiler flags (-D tunables), `out` names another output file."""
    lib = out or LIB
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + (extra or []) + ["-o", tmp, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature name; that note is harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed building libmmvseg.so")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
