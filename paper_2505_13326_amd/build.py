"""Builds libsart.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_DIR = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_DIR)
CSRC = os.path.join(_DIR, "csrc")
LIB = os.path.join(_DIR, "libsart.so")
SOURCES = ["sart_api.hip", "sart_bookkeeping.hip", "sart_attention.hip", "sart_prefill.hip", "sart_probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(_ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, extra_flags=(), out: str = LIB, obj_dir: str = CSRC) -> str:
    """Compiles every source (always; no staleness check) and links the library."""
    objs = []
    os.makedirs(obj_dir, exist_ok=True)

    def one(src):
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = ["hipcc", "-c", *FLAGS, *extra_flags, os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
