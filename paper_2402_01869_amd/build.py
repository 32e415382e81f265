"""Compile the HIP library for gfx950 into paper_2402_01869_amd/libinfercept_hot.so (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libinfercept_hot.so")
SOURCES = ["ic_api.hip", "kv_swap.hip", "swap_pipe.hip", "waste_model.hip", "attn_row.hip", "attn_tile.hip", "attn_group.hip", "attn_group_slim.hip",
           "ceilings.hip"]
HEADERS = [os.path.join(CSRC, "ic_internal.h"), os.path.join(CSRC, "row_body.h"), os.path.join(CSRC, "tile_body.h"), os.path.join(CSRC, "tile16_body.h"),
           os.path.join(os.path.dirname(HERE), "include", "infercept_hot.h"),
           os.path.join(os.path.dirname(HERE), "include", "infercept_measure.h")]

# Packed-fp32 VALU forms are disabled on purpose (hipcc only; the host pass warns and ignores it).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    cmd = ["hipcc"] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and r.stderr:
        sys.stderr.write(r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
