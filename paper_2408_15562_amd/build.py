"""Builds libfspad.so (HIP, gfx950) in-tree with hipcc: one object per source, compiled side by side, then linked."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libfspad.so")
ROOFS_LIB_PATH = os.path.join(_HERE, "libfspad_roofs.so")   # the benchmark's measurement kernels, not the product
OBJ_DIR = os.path.join(_HERE, "_build")
SOURCES = ["fspad_host.cpp", "fspad_attn.hip", "fspad_accept.hip", "fspad_commit.hip", "fspad_tree.hip", "fspad_lmhead.hip",
           "fspad_topk.hip", "fspad_draft.hip"]
HEADERS = ["greedy_walk.h", "stream_gemm.h", "exp_nonpos.h"]

_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          # packed fp32 VALU ops are kept off on the test machines
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(_ROOT, "include")]


# per-source options. The attention kernels keep the results of their matrix instructions in ordinary
# vector registers: left to itself the compiler puts the score tiles into accumulation registers and
# copies every one of them out again for the softmax (a quarter of the instructions of a block).
EXTRA_FLAGS = {"fspad_attn.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def compile_command(src: str, obj: str, defines=()):
    return (["hipcc", "-c"] + _FLAGS + EXTRA_FLAGS.get(src, []) + [f"-D{d}" for d in defines]
            + ["-o", obj, os.path.join(CSRC, src)])


def link_command(objs, out: str = LIB_PATH):
    return ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + list(objs)


def _deps():
    return ([os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(CSRC, h) for h in HEADERS if os.path.exists(os.path.join(CSRC, h))]
            + [os.path.join(_ROOT, "include", "fspad.h")])


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(d) > built for d in _deps())


def build(force: bool = True, verbose: bool = False, defines=(), out: str = LIB_PATH, only_changed: bool = False) -> str:
    """Compile the library. `force=False` rebuilds only when a source is newer than the library.
    `only_changed=True` recompiles only the objects whose source (or any header) is newer than the object."""
    if not (force or is_stale()):
        return out
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = "_".join(defines)
    hdr_time = max(os.path.getmtime(d) for d in _deps() if d.endswith(".h"))

    def one(src):
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + (f".{tag}" if tag else "") + ".o")
        if only_changed and os.path.exists(obj) and os.path.getmtime(obj) > max(hdr_time, os.path.getmtime(os.path.join(CSRC, src))):
            return obj, ""
        proc = subprocess.run(compile_command(src, obj, defines), capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + proc.stdout + proc.stderr)
        return obj, proc.stderr

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        results = list(pool.map(one, SOURCES))
    proc = subprocess.run(link_command([o for o, _ in results], out), capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stdout + proc.stderr)
    if out == LIB_PATH:
        build_roofs(force=not only_changed)
    if verbose:
        print("".join(log for _, log in results) + proc.stderr)
    return out


def build_roofs(force: bool = True) -> str:
    """The benchmark's roof kernels (plain read, copy, matrix-core loop): a library of their own."""
    src = os.path.join(CSRC, "bench_roofs.hip")
    if not force and os.path.exists(ROOFS_LIB_PATH) and os.path.getmtime(ROOFS_LIB_PATH) > os.path.getmtime(src):
        return ROOFS_LIB_PATH
    proc = subprocess.run(["hipcc"] + _FLAGS + ["-shared", "-o", ROOFS_LIB_PATH, src], capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on bench_roofs.hip:\n" + proc.stdout + proc.stderr)
    return ROOFS_LIB_PATH


if __name__ == "__main__":
    import sys
    print(build(force=True, verbose="-v" in sys.argv, only_changed="--changed" in sys.argv))
