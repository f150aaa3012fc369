"""Builds `liblsq.so` (the C-ABI library of include/lsq.h) for gfx950 with hipcc.

    python -m paper_2110_05722_amd.build

hipcc cross-compiles without a GPU.  Each translation unit is compiled on its
own (in parallel) and the objects are linked into one shared library that sits
next to this file, so it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblsq.so")
OBJ_DIR = os.path.join(HERE, "_build", "liblsq.so")
SOURCES = ["api", "calibrate", "adam", "bias_dropout_residual", "bias_act_dropout", "heads", "embedding", "pad", "layernorm", "softmax",
           "ls_xent"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are switched off for the device pass (the host pass warns that it
    # does not know the feature; that is harmless)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(name: str, obj_dir: str = OBJ_DIR, extra: tuple = ()) -> str:
    src = os.path.join(CSRC, name + ".hip")
    obj = os.path.join(obj_dir, name + ".o")
    r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    noise = ("packed-fp32-ops", "1 warning generated")
    err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in noise))
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}.hip:\n{r.stderr}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, lib: str = LIB, obj_dir: str = OBJ_DIR, extra: tuple = ()) -> str:
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda n: _compile(n, obj_dir, extra), SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True,
                   capture_output=not verbose)
    if verbose:
        print(f"built {lib}")
    return lib


if __name__ == "__main__":
    build()
