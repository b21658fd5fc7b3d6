"""Compile libssrnn.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_1803_11389_amd.build

Every kernel family is a translation unit of its own; they are compiled side by
side (at most 8 at a time) into _build/ and linked into one shared library.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssrnn.so")
SOURCES = [
    "ssrnn.hip", "launch_valu.hip", "launch_mfma_lds.hip",
    "launch_mfma_packed_f32.hip", "launch_mfma_packed_bf16.hip", "launch_mfma_packed_fp8.hip",
    "launch_mfma_xlds_f32.hip", "launch_mfma_xlds_bf16.hip", "launch_mfma_xlds_fp8.hip", "launch_lstm.hip",
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of every kernel on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, extra_flags=(), only=None) -> str:
    """Compiles every source (or those named in `only`; the other objects must exist) and links."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"{src}: hipcc failed\n{out}")
        if out.strip():
            print(out, flush=True)
        return obj

    todo = [s for s in SOURCES if only is None or s in only]
    with ThreadPoolExecutor(max_workers=min(8, len(todo))) as ex:
        list(ex.map(compile_one, todo))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if a.startswith("-")]
    only = [a for a in sys.argv[1:] if not a.startswith("-")] or None
    build(verbose=True, extra_flags=flags, only=only)
