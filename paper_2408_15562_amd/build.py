"""Builds libfspad.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libfspad.so")
SOURCES = ["fspad_host.cpp", "fspad_attn.hip", "fspad_accept.hip", "fspad_commit.hip", "fspad_tree.hip", "fspad_lmhead.hip", "fspad_topk.hip", "fspad_draft.hip"]


def hipcc_command(out: str = LIB_PATH):
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
            # packed fp32 VALU ops are kept off on the test machines
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I", os.path.join(_ROOT, "include"), "-o", out] + srcs


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, s) for s in SOURCES + ["greedy_walk.h", "stream_gemm.h", "exp_nonpos.h"]] + [os.path.join(_ROOT, "include", "fspad.h")]
    return any(os.path.getmtime(d) > built for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library. `force=False` rebuilds only when a source is newer."""
    if force or is_stale():
        proc = subprocess.run(hipcc_command(), capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
        if verbose:
            print(proc.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True, verbose=True))
