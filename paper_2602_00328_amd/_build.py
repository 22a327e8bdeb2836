"""Builds libharvest.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libharvest.so")
SOURCES = [os.path.join(HERE, "csrc", "harvest.hip")]
HEADERS = [os.path.join(HERE, "csrc", "kernels.h"), os.path.join(os.path.dirname(HERE), "include", "harvest.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return LIB_PATH


def library_is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


EXAMPLE_SRC = os.path.join(HERE, "examples", "kv_fetch.c")
EXAMPLE_BIN = os.path.join(HERE, "examples", "kv_fetch")


def build_example() -> str:
    """The plain-C user of the ABI (no Python in its process); links the library built above."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O1", "-Wno-unused-command-line-argument", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-I", os.path.join(os.path.dirname(HERE), "include"), EXAMPLE_SRC, "-x", "none",
           "-o", EXAMPLE_BIN, "-L", HERE, "-l:libharvest.so", "-Wl,-rpath,$ORIGIN/.."]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on the example ({res.returncode}):\n{res.stderr}")
    return EXAMPLE_BIN
